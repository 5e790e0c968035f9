"""Thin ctypes binding of libsalus.so (C ABI in include/salus.h).

Argument marshalling only: every step of the path runs inside the library.
There is no fallback: if the library is missing, loading raises.
"""
import ctypes as C
import os

import torch  # noqa: F401  (first, so that the HIP runtime already loaded by torch is the one the library binds to)

_HERE = os.path.dirname(os.path.abspath(__file__))
# SALUS_LIBRARY names another build of the same sources (the sanitizer build of the tests)
LIB_PATH = os.environ.get("SALUS_LIBRARY") or os.path.join(_HERE, "libsalus.so")

OK, QUEUED = 0, 1
EINVAL, ENOMEM, ENOTRESIDENT, EBUSY, ENEVER, EHIP, ETIMEOUT = -1, -2, -3, -4, -5, -6, -7
POLICY_FIFO, POLICY_FAIR, POLICY_PRIORITY, POLICY_PACK = 0, 1, 2, 3
JOB_QUEUED, JOB_RESIDENT, JOB_EVICTED, JOB_DONE = 0, 1, 2, 3
ACT_NONE, ACT_RELU, ACT_GELU = 0, 1, 2
F32, BF16 = 0, 1
COPY_KERNEL, COPY_DMA = 0, 1
LAYOUT_ROWMAJOR, LAYOUT_STRIP128 = 0, 1
FLAG_SHRINK_LANES = 1
FLAG_FUSE_DEPTHS = 2


class Config(C.Structure):
    _fields_ = [("granule", C.c_uint64), ("max_lanes", C.c_uint32), ("policy", C.c_int32),
                ("stream", C.c_void_p), ("copy_engine", C.c_int32), ("flags", C.c_uint32)]


class JobInfo(C.Structure):
    _fields_ = [("state", C.c_int32), ("lane", C.c_int32), ("priority", C.c_int32),
                ("auto_evicted", C.c_int32), ("in_transit", C.c_int32), ("lane_parked", C.c_int32),
                ("P", C.c_uint64), ("E", C.c_uint64),
                ("persist_off", C.c_uint64), ("lane_off", C.c_uint64), ("lane_size", C.c_uint64),
                ("pending", C.c_uint64), ("served", C.c_uint64),
                ("cost", C.c_uint64), ("attained", C.c_uint64),
                ("arrival_round", C.c_uint64), ("admit_round", C.c_uint64)]


class Slot(C.Structure):
    _fields_ = [("job", C.c_int32), ("lane", C.c_int32)]


class Move(C.Structure):
    _fields_ = [("src", C.c_uint64), ("dst", C.c_uint64), ("len", C.c_uint64)]


class Layer(C.Structure):
    _fields_ = [("K", C.c_uint32), ("N", C.c_uint32), ("w_off", C.c_uint64),
                ("act", C.c_int32), ("layout", C.c_int32)]


class GemmDesc(C.Structure):
    _fields_ = [("job", C.c_int32), ("M", C.c_uint32), ("n_layers", C.c_uint32),
                ("dtype", C.c_int32), ("layers", C.POINTER(Layer)),
                ("x_off", C.c_uint64), ("y_off", C.c_uint64), ("h_off", C.c_uint64)]


class TrainLayer(C.Structure):
    _fields_ = [("K", C.c_uint32), ("N", C.c_uint32), ("wb_off", C.c_uint64), ("wm_off", C.c_uint64)]


class TrainDesc(C.Structure):
    _fields_ = [("job", C.c_int32), ("M", C.c_uint32), ("n_layers", C.c_uint32), ("lr", C.c_float),
                ("layers", C.POINTER(TrainLayer)),
                ("x_off", C.c_uint64), ("labels_off", C.c_uint64), ("logits_off", C.c_uint64),
                ("loss_off", C.c_uint64), ("work_off", C.c_uint64)]


class Stats(C.Structure):
    _fields_ = [(n, C.c_uint64) for n in (
        "rounds", "iterations", "bytes_d2h", "bytes_h2d", "bytes_d2d", "moves", "compactions",
        "lanes_opened", "lanes_deleted", "lanes_moved", "evictions", "restores", "admitted",
        "queued", "gemm_launches", "fused_timeouts")]


class Event(C.Structure):
    _fields_ = [("kind", C.c_int32), ("pad", C.c_int32), ("a", C.c_uint64), ("b", C.c_uint64)]


_PROTOS = {
    "salus_pool_create": [C.c_void_p, C.c_uint64, C.POINTER(Config), C.POINTER(C.c_void_p)],
    "salus_pool_destroy": [C.c_void_p],
    "salus_lane_alloc": [C.c_void_p, C.c_uint64, C.c_uint64, C.c_int32, C.c_uint64,
                         C.POINTER(C.c_int32)],
    "salus_lane_free": [C.c_void_p, C.c_int32],
    "salus_job_query": [C.c_void_p, C.c_int32, C.POINTER(JobInfo)],
    "salus_job_set_pending": [C.c_void_p, C.c_int32, C.c_uint64],
    "salus_job_set_cost": [C.c_void_p, C.c_int32, C.c_uint64],
    "salus_fused_check": [C.c_void_p],
    "salus_fused_spin_limit": [C.c_void_p, C.c_uint32],
    "salus_compact_spin_limit": [C.c_void_p, C.c_uint32],
    "salus_set_pending_many": [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_uint64), C.c_uint32],
    "salus_job_write": [C.c_void_p, C.c_int32, C.c_uint64, C.c_void_p, C.c_uint64],
    "salus_job_read": [C.c_void_p, C.c_int32, C.c_uint64, C.c_void_p, C.c_uint64],
    "salus_schedule_iteration": [C.c_void_p, C.POINTER(Slot), C.c_uint32, C.POINTER(C.c_uint32)],
    "salus_grouped_forward": [C.c_void_p, C.POINTER(GemmDesc), C.c_uint32, C.c_void_p],
    "salus_grouped_forward_static": [C.c_void_p, C.POINTER(GemmDesc), C.c_uint32, C.c_void_p],
    "salus_train_work_bytes": [C.c_uint32, C.POINTER(TrainLayer), C.c_uint32],
    "salus_forward_work_bytes": [C.c_uint32, C.POINTER(Layer), C.c_uint32, C.c_int32],
    "salus_grouped_train_step": [C.c_void_p, C.POINTER(TrainDesc), C.c_uint32, C.c_void_p],
    "salus_switch_out": [C.c_void_p, C.c_int32, C.c_void_p],
    "salus_switch_in": [C.c_void_p, C.c_int32],
    "salus_switch_out_begin": [C.c_void_p, C.c_int32, C.c_void_p, C.c_void_p],
    "salus_switch_out_end": [C.c_void_p, C.c_int32, C.c_int32],
    "salus_switch_in_begin": [C.c_void_p, C.c_int32, C.c_void_p],
    "salus_switch_in_end": [C.c_void_p, C.c_int32, C.c_int32],
    "salus_compact": [C.c_void_p, C.POINTER(Move), C.c_uint32, C.POINTER(C.c_uint32)],
    "salus_get_stats": [C.c_void_p, C.POINTER(Stats)],
    "salus_poll_events": [C.c_void_p, C.POINTER(Event), C.c_uint32, C.POINTER(C.c_uint32)],
    "salus_lanes": [C.c_void_p, C.POINTER(C.c_int32), C.POINTER(C.c_uint64), C.POINTER(C.c_uint64),
                    C.c_uint32, C.POINTER(C.c_uint32)],
    "salus_last_error": [C.c_void_p],
    "salus_scan_u64": [C.c_void_p, C.c_uint32, C.c_void_p, C.c_void_p, C.c_void_p],
    "salus_fill_pattern": [C.c_void_p, C.c_uint64, C.c_uint64, C.c_void_p],
    "salus_check_pattern": [C.c_void_p, C.c_uint64, C.c_uint64, C.c_void_p, C.POINTER(C.c_uint64),
                            C.c_void_p],
    "salus_copy": [C.c_void_p, C.c_void_p, C.c_uint64, C.c_void_p],
    "salus_calibrate_mfma": [C.c_void_p, C.c_uint32, C.c_int32, C.c_void_p, C.POINTER(C.c_uint64)],
    "salus_calibrate_read": [C.c_void_p, C.c_uint64, C.c_void_p, C.c_void_p],
    "salus_pack_strip128": [C.c_void_p, C.c_void_p, C.c_uint32, C.c_uint32],
}

_lib = None


def lib():
    """The loaded library; raises if it has not been built."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(
                f"{LIB_PATH} is missing: build it with `python -m paper_1902_04610_amd.build` "
                "(there is no fallback path)")
        L = C.CDLL(LIB_PATH)
        for name, args in _PROTOS.items():
            fn = getattr(L, name)
            fn.argtypes = args
            fn.restype = (C.c_char_p if name == "salus_last_error" else
                          C.c_uint64 if name.endswith("_work_bytes") else C.c_int32)
        _lib = L
    return _lib


class SalusError(RuntimeError):
    def __init__(self, code, msg):
        super().__init__(f"salus error {code}: {msg}")
        self.code = code


class Pool:
    """One pool = one caller-owned device range.  Methods mirror the C calls
    one to one and return plain Python values."""

    def __init__(self, base_ptr, capacity, granule=256, max_lanes=0, policy=POLICY_FAIR,
                 stream=None, copy_engine=COPY_KERNEL, shrink_lanes=False, fuse_depths=False):
        self._lib = lib()
        cfg = Config(granule, max_lanes, policy, stream, copy_engine,
                     (FLAG_SHRINK_LANES if shrink_lanes else 0) | (FLAG_FUSE_DEPTHS if fuse_depths else 0))
        h = C.c_void_p()
        rc = self._lib.salus_pool_create(base_ptr, capacity, C.byref(cfg), C.byref(h))
        if rc != OK:
            raise SalusError(rc, "salus_pool_create rejected its arguments")
        self._h = h
        self.capacity = capacity

    def close(self):
        if self._h:
            self._lib.salus_pool_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def _check(self, rc, allowed=(OK,)):
        if rc not in allowed:
            raise SalusError(rc, (self._lib.salus_last_error(self._h) or b"").decode())
        return rc

    def last_error(self):
        return (self._lib.salus_last_error(self._h) or b"").decode()

    # -- Algorithm 1 ---------------------------------------------------------
    def lane_alloc(self, P, E, priority=0, pending=0):
        """Returns (status, job id); status may be OK, QUEUED, ENEVER or EINVAL."""
        job = C.c_int32(-1)
        rc = self._lib.salus_lane_alloc(self._h, P, E, priority, pending, C.byref(job))
        self._check(rc, (OK, QUEUED, ENEVER, EINVAL))
        return rc, job.value

    def lane_free(self, job):
        return self._lib.salus_lane_free(self._h, job)

    def job_query(self, job):
        info = JobInfo()
        self._check(self._lib.salus_job_query(self._h, job, C.byref(info)))
        return info

    def job_set_pending(self, job, n):
        return self._lib.salus_job_set_pending(self._h, job, n)

    def job_set_cost(self, job, cost):
        return self._lib.salus_job_set_cost(self._h, job, cost)

    def fused_check(self):
        return self._lib.salus_fused_check(self._h)

    def fused_spin_limit(self, polls):
        return self._lib.salus_fused_spin_limit(self._h, polls)

    def compact_spin_limit(self, polls):
        return self._lib.salus_compact_spin_limit(self._h, polls)

    def set_pending_many(self, jobs_arr, n_arr, count):
        """jobs_arr: ctypes int32 array, n_arr: ctypes uint64 array."""
        return self._lib.salus_set_pending_many(self._h, jobs_arr, n_arr, count)

    def job_write(self, job, off, host_ptr, nbytes):
        self._check(self._lib.salus_job_write(self._h, job, off, host_ptr, nbytes))

    def job_read(self, job, off, host_ptr, nbytes):
        self._check(self._lib.salus_job_read(self._h, job, off, host_ptr, nbytes))

    def lanes(self):
        n = C.c_uint32()
        self._lib.salus_lanes(self._h, None, None, None, 0, C.byref(n))
        k = n.value
        ids, offs, sizes = (C.c_int32 * k)(), (C.c_uint64 * k)(), (C.c_uint64 * k)()
        self._lib.salus_lanes(self._h, ids, offs, sizes, k, C.byref(n))
        return [(ids[i], offs[i], sizes[i]) for i in range(k)]

    # -- scheduling ------------------------------------------------------------
    def schedule_iteration(self, cap=256):
        slots = (Slot * cap)()
        n = C.c_uint32()
        self._check(self._lib.salus_schedule_iteration(self._h, slots, cap, C.byref(n)))
        return [(slots[i].job, slots[i].lane) for i in range(n.value)]

    def schedule_into(self, slots, cap):
        """Allocation-free variant: fills a caller-owned Slot array, returns the count."""
        n = C.c_uint32()
        self._check(self._lib.salus_schedule_iteration(self._h, slots, cap, C.byref(n)))
        return n.value

    # -- packed iteration --------------------------------------------------------
    @staticmethod
    def make_descs(items):
        """items: iterable of dicts(job, M, dtype, layers=[(K, N, w_off, act[, layout])], x_off,
        y_off, h_off).  Returns (array, keepalive) ready for grouped_forward."""
        items = list(items)
        arr = (GemmDesc * len(items))()
        keep = []
        for i, it in enumerate(items):
            L = (Layer * len(it["layers"]))(*[Layer(t[0], t[1], t[2], t[3], t[4] if len(t) > 4 else 0)
                                              for t in it["layers"]])
            keep.append(L)
            arr[i] = GemmDesc(it["job"], it["M"], len(it["layers"]), it["dtype"], L,
                              it["x_off"], it["y_off"], it.get("h_off", 0))
        return arr, keep

    def grouped_forward(self, descs, n=None, stream=None):
        if n is None:
            n = len(descs)
        return self._check(self._lib.salus_grouped_forward(self._h, descs, n, stream),
                           (OK, EINVAL, ENOTRESIDENT, EBUSY))

    def grouped_forward_static(self, descs, n=None, stream=None):
        if n is None:
            n = len(descs)
        return self._check(self._lib.salus_grouped_forward_static(self._h, descs, n, stream),
                           (OK, EINVAL, ENOTRESIDENT, EBUSY, ENOMEM))

    @staticmethod
    def make_train_descs(items):
        """items: dicts(job, M, lr, layers=[(K, N, wb_off, wm_off)], x_off, labels_off,
        logits_off, loss_off, work_off)."""
        items = list(items)
        arr = (TrainDesc * len(items))()
        keep = []
        for i, it in enumerate(items):
            L = (TrainLayer * len(it["layers"]))(*[TrainLayer(*t) for t in it["layers"]])
            keep.append(L)
            arr[i] = TrainDesc(it["job"], it["M"], len(it["layers"]), it["lr"], L, it["x_off"],
                               it["labels_off"], it["logits_off"], it["loss_off"], it["work_off"])
        return arr, keep

    def grouped_train_step(self, descs, n=None, stream=None):
        if n is None:
            n = len(descs)
        return self._check(self._lib.salus_grouped_train_step(self._h, descs, n, stream),
                           (OK, EINVAL, ENOTRESIDENT, EBUSY))

    # -- switching -----------------------------------------------------------------
    def switch_out(self, job, pinned_ptr=None):
        return self._lib.salus_switch_out(self._h, job, pinned_ptr)

    def switch_in(self, job):
        return self._lib.salus_switch_in(self._h, job)

    def switch_out_begin(self, job, copy_stream, pinned_ptr=None):
        return self._lib.salus_switch_out_begin(self._h, job, pinned_ptr, copy_stream)

    def switch_out_end(self, job, wait=True):
        return self._lib.salus_switch_out_end(self._h, job, 1 if wait else 0)

    def switch_in_begin(self, job, copy_stream):
        return self._lib.salus_switch_in_begin(self._h, job, copy_stream)

    def switch_in_end(self, job, wait=True):
        return self._lib.salus_switch_in_end(self._h, job, 1 if wait else 0)

    def compact(self, cap=4096):
        plan = (Move * cap)()
        n = C.c_uint32()
        self._check(self._lib.salus_compact(self._h, plan, cap, C.byref(n)))
        return [(plan[i].src, plan[i].dst, plan[i].len) for i in range(min(n.value, cap))]

    # -- introspection ----------------------------------------------------------------
    def stats(self):
        s = Stats()
        self._lib.salus_get_stats(self._h, C.byref(s))
        return {n: getattr(s, n) for n, _ in Stats._fields_}

    def poll_events(self, cap=65536):
        ev = (Event * cap)()
        n = C.c_uint32()
        self._lib.salus_poll_events(self._h, ev, cap, C.byref(n))
        return [(ev[i].kind, ev[i].a, ev[i].b) for i in range(n.value)]


def forward_work_bytes(M, layers, dtype):
    """layers: [(K, N, w_off, act)]"""
    L = (Layer * len(layers))(*[Layer(t[0], t[1], t[2], t[3], 0) for t in layers])
    return lib().salus_forward_work_bytes(M, L, len(layers), dtype)


def train_work_bytes(M, layers):
    """layers: [(K, N, wb_off, wm_off)]"""
    L = (TrainLayer * len(layers))(*[TrainLayer(*t) for t in layers])
    return lib().salus_train_work_bytes(M, L, len(layers))


def scan_u64(values, scratch_ptr, stream=None):
    n = len(values)
    a = (C.c_uint64 * n)(*values)
    out = (C.c_uint64 * (n + 1))()
    rc = lib().salus_scan_u64(a, n, out, scratch_ptr, stream)
    if rc != OK:
        raise SalusError(rc, "salus_scan_u64")
    return list(out)


def fill_pattern(dev_ptr, nbytes, seed, stream=None):
    rc = lib().salus_fill_pattern(dev_ptr, nbytes, seed, stream)
    if rc != OK:
        raise SalusError(rc, "salus_fill_pattern")


def check_pattern(dev_ptr, nbytes, seed, scratch_ptr, stream=None):
    bad = C.c_uint64()
    rc = lib().salus_check_pattern(dev_ptr, nbytes, seed, scratch_ptr, C.byref(bad), stream)
    if rc != OK:
        raise SalusError(rc, "salus_check_pattern")
    return bad.value


def pack_strip128(w):
    """K x N uint16 (bf16 bits) numpy array, row-major -> the same values in
    LAYOUT_STRIP128 order (a new flat array of K * N elements)."""
    import numpy as np
    w = np.ascontiguousarray(w, dtype=np.uint16)
    out = np.empty(w.size, np.uint16)
    rc = lib().salus_pack_strip128(w.ctypes.data, out.ctypes.data, w.shape[0], w.shape[1])
    if rc != OK:
        raise SalusError(rc, "salus_pack_strip128")
    return out


def copy(dst_ptr, src_ptr, nbytes, stream=None):
    rc = lib().salus_copy(dst_ptr, src_ptr, nbytes, stream)
    if rc != OK:
        raise SalusError(rc, "salus_copy")


def calibrate_mfma(dev_out_ptr, slabs, from_lds, stream=None):
    """Launches the matrix-pipe calibration kernel; returns the launch's flop count."""
    flop = C.c_uint64()
    rc = lib().salus_calibrate_mfma(dev_out_ptr, slabs, 1 if from_lds else 0, stream, C.byref(flop))
    if rc != OK:
        raise SalusError(rc, "salus_calibrate_mfma")
    return flop.value


def calibrate_read(dev_ptr, nbytes, sink_ptr, stream=None):
    """Launches the load-only calibration kernel over [dev_ptr, dev_ptr + nbytes)."""
    rc = lib().salus_calibrate_read(dev_ptr, nbytes, sink_ptr, stream)
    if rc != OK:
        raise SalusError(rc, "salus_calibrate_read")
