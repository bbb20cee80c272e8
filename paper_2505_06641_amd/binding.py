"""ctypes binding of the C ABI in include/sneakpeek.h.

Argument marshalling only: every step of the path runs in the HIP library.
PyTorch is used for device memory and streams.  There is no CPU fallback: if
the library has not been built, loading raises.
"""
from __future__ import annotations

import ctypes as C
import os
from typing import Optional

import numpy as np

_PKG = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.path.join(_PKG, "libsneakpeek_hip.so")

SP_OK, SP_DONE = 0, 1
SP_EINVAL, SP_ENOMEM, SP_EDEVICE, SP_ESTATE, SP_ECAPACITY = -1, -2, -3, -4, -5
SP_DUMP_ORDER, SP_DUMP_SEGMENTS, SP_DUMP_SCORE_CUBE, SP_DUMP_LOGITS = 0, 1, 2, 3

EXPORTS = ["sp_create", "sp_destroy", "sp_score", "sp_greedy_round", "sp_greedy_round_static", "sp_schedule", "sp_debug_dump",
           "sp_strerror", "sp_last_hip_error", "sp_max_models", "sp_max_classes",
           "sp_rounds_in_one_launch", "sp_debug_mfma_rate", "sp_debug_copy_rate", "sp_debug_set_generation", "sp_debug_set_spin_limit", "sp_debug_set_sort_spin_limit", "sp_set_prior", "sp_set_swap_cost", "sp_set_policy",
           "sp_set_timing", "sp_get_timing", "sp_get_round_times"]


class sp_policy(C.Structure):
    _fields_ = [("order", C.c_int32), ("select", C.c_int32), ("batch_rule", C.c_int32), ("choice", C.c_int32),
                ("weight", C.c_int32), ("batch_cap", C.c_int32), ("split_groups", C.c_int32)]


class sp_profile(C.Structure):
    _fields_ = [
        ("n_apps", C.c_int32), ("feat_dim", C.c_int32), ("hidden_dim", C.c_int32), ("max_batch", C.c_int32),
        ("feat_dtype", C.c_int32), ("max_requests", C.c_int32),
        ("n_classes", C.POINTER(C.c_int32)), ("n_models", C.POINTER(C.c_int32)),
        ("W1", C.POINTER(C.c_void_p)), ("b1", C.POINTER(C.c_void_p)),
        ("W2", C.POINTER(C.c_void_p)), ("b2", C.POINTER(C.c_void_p)),
        ("acc", C.POINTER(C.c_void_p)), ("lat_ms", C.POINTER(C.c_void_p)),
        ("penalty", C.POINTER(C.c_int32)), ("prio_timescale_ms", C.c_float),
    ]


class sp_decision(C.Structure):
    _fields_ = [("app", C.c_int32), ("model", C.c_int32), ("batch", C.c_int32), ("round", C.c_int32),
                ("t_start_ms", C.c_double), ("t_end_ms", C.c_double),
                ("score", C.c_float), ("batch_utility", C.c_float)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class sp_summary(C.Structure):
    _fields_ = [("total_weighted_utility", C.c_double), ("mean_utility", C.c_double),
                ("total_violation_ms", C.c_double), ("n_rounds", C.c_int32), ("n_scheduled", C.c_int32),
                ("n_dropped", C.c_int32), ("done", C.c_int32)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


class sp_timing(C.Structure):
    _fields_ = [("group_ms", C.c_float), ("score_kernel_ms", C.c_float), ("order_ms", C.c_float),
                ("rounds_ms", C.c_float), ("n_rounds_timed", C.c_int32), ("finish_order_ms", C.c_float),
                ("copy_outputs_ms", C.c_float), ("utility_evaluations", C.c_int64)]

    def as_dict(self):
        return {k: getattr(self, k) for k, _ in self._fields_}


_lib = None


def load_library(path: Optional[str] = None):
    """Load the HIP library (torch first, so that both share one HIP runtime)."""
    global _lib
    if _lib is not None and path is None:
        return _lib
    import torch  # noqa: F401  (brings in libamdhip64 with the soname the library links against)
    p = path or LIB_PATH
    if not os.path.exists(p):
        raise RuntimeError(f"{p} is missing: build it first (python -m paper_2505_06641_amd.build)")
    lib = C.CDLL(p)
    vp, i32p = C.c_void_p, C.c_void_p
    lib.sp_create.argtypes = [C.POINTER(sp_profile), C.c_int, C.POINTER(vp)]
    lib.sp_create.restype = C.c_int
    lib.sp_destroy.argtypes = [vp]
    lib.sp_destroy.restype = None
    lib.sp_score.argtypes = [vp, C.c_int32, vp, i32p, vp, vp, vp, vp, vp]
    lib.sp_score.restype = C.c_int
    lib.sp_greedy_round.argtypes = [vp, vp, C.POINTER(sp_decision), i32p]
    lib.sp_greedy_round.restype = C.c_int
    lib.sp_greedy_round_static.argtypes = [vp, vp, C.POINTER(sp_decision), i32p]
    lib.sp_greedy_round_static.restype = C.c_int
    lib.sp_schedule.argtypes = [vp, C.c_int32, vp, i32p, i32p, i32p, vp, C.POINTER(sp_decision), C.c_int32,
                                C.POINTER(sp_summary)]
    lib.sp_schedule.restype = C.c_int
    lib.sp_debug_dump.argtypes = [vp, C.c_int32, vp, vp, i32p, vp]
    lib.sp_debug_dump.restype = C.c_int
    lib.sp_strerror.argtypes = [C.c_int]
    lib.sp_strerror.restype = C.c_char_p
    lib.sp_last_hip_error.argtypes = [vp]
    lib.sp_last_hip_error.restype = C.c_char_p
    lib.sp_max_models.argtypes = [vp]
    lib.sp_max_models.restype = C.c_int32
    lib.sp_max_classes.argtypes = [vp]
    lib.sp_max_classes.restype = C.c_int32
    lib.sp_set_prior.argtypes = [vp, C.c_int32, C.c_void_p, C.c_float]
    lib.sp_set_prior.restype = C.c_int
    lib.sp_set_policy.argtypes = [vp, C.POINTER(sp_policy)]
    lib.sp_set_policy.restype = C.c_int
    lib.sp_set_swap_cost.argtypes = [vp, C.c_int32, C.c_void_p]
    lib.sp_set_swap_cost.restype = C.c_int
    lib.sp_rounds_in_one_launch.argtypes = [vp]
    lib.sp_rounds_in_one_launch.restype = C.c_int32
    lib.sp_debug_set_generation.argtypes = [vp, C.c_uint32]
    lib.sp_debug_set_generation.restype = C.c_int
    lib.sp_debug_set_spin_limit.argtypes = [vp, C.c_int32]
    lib.sp_debug_set_spin_limit.restype = C.c_int
    lib.sp_debug_set_sort_spin_limit.argtypes = [vp, C.c_int32]
    lib.sp_debug_set_sort_spin_limit.restype = C.c_int
    lib.sp_debug_mfma_rate.argtypes = [C.c_int, C.c_int32, C.c_int32, C.c_int32, vp, C.POINTER(C.c_double), C.POINTER(C.c_double)]
    lib.sp_debug_mfma_rate.restype = C.c_int
    lib.sp_debug_copy_rate.argtypes = [C.c_int, C.c_int64, vp, C.POINTER(C.c_double)]
    lib.sp_debug_copy_rate.restype = C.c_int
    lib.sp_set_timing.argtypes = [vp, C.c_int32]
    lib.sp_set_timing.restype = C.c_int
    lib.sp_get_timing.argtypes = [vp, C.POINTER(sp_timing)]
    lib.sp_get_timing.restype = C.c_int
    lib.sp_get_round_times.argtypes = [vp, C.POINTER(C.c_float), C.c_int32, C.POINTER(C.c_int32)]
    lib.sp_get_round_times.restype = C.c_int
    if path is None:
        _lib = lib
    return lib


class SneakPeekError(RuntimeError):
    def __init__(self, status, where, detail=""):
        self.status = status
        super().__init__(f"{where}: status {status} ({detail})")


def _ptr_array(arrays):
    arr = (C.c_void_p * len(arrays))()
    for i, a in enumerate(arrays):
        arr[i] = None if a is None else a.ctypes.data
    return arr


def marshal_profile(profile, max_requests: int):
    """Build the C struct; returns (struct, keepalive list)."""
    A = int(profile.n_apps)
    wdt = np.uint16 if profile.feat_dtype == 1 else np.float32
    keep = []

    def c_arr(a, dt):
        b = np.ascontiguousarray(a, dtype=dt)
        keep.append(b)
        return b

    ncls = c_arr(profile.n_classes, np.int32)
    nmod = c_arr(profile.n_models, np.int32)
    pen = c_arr(profile.penalty, np.int32)
    W1 = [c_arr(w, wdt) for w in profile.W1]
    b1 = [c_arr(b, np.float32) for b in profile.b1]
    has2 = int(profile.hidden_dim) > 0
    W2 = [c_arr(w, wdt) for w in profile.W2] if has2 else None
    b2 = [c_arr(b, np.float32) for b in profile.b2] if has2 else None
    acc = [c_arr(a, np.float32) for a in profile.acc]
    lat = [c_arr(l, np.float32) for l in profile.lat_ms]
    ps = [_ptr_array(W1), _ptr_array(b1), _ptr_array(W2) if has2 else None, _ptr_array(b2) if has2 else None,
          _ptr_array(acc), _ptr_array(lat)]
    keep.extend(ps)
    s = sp_profile()
    s.n_apps, s.feat_dim, s.hidden_dim = A, int(profile.feat_dim), int(profile.hidden_dim)
    s.max_batch, s.feat_dtype, s.max_requests = int(profile.max_batch), int(profile.feat_dtype), int(max_requests)
    s.n_classes = ncls.ctypes.data_as(C.POINTER(C.c_int32))
    s.n_models = nmod.ctypes.data_as(C.POINTER(C.c_int32))
    s.penalty = pen.ctypes.data_as(C.POINTER(C.c_int32))
    s.W1 = C.cast(ps[0], C.POINTER(C.c_void_p))
    s.b1 = C.cast(ps[1], C.POINTER(C.c_void_p))
    s.W2 = C.cast(ps[2], C.POINTER(C.c_void_p)) if has2 else None
    s.b2 = C.cast(ps[3], C.POINTER(C.c_void_p)) if has2 else None
    s.acc = C.cast(ps[4], C.POINTER(C.c_void_p))
    s.lat_ms = C.cast(ps[5], C.POINTER(C.c_void_p))
    s.prio_timescale_ms = float(profile.prio_timescale_ms)
    return s, keep


def _dptr(t):
    return None if t is None else C.c_void_p(t.data_ptr())


def _stream_ptr(stream):
    if stream is None:
        import torch
        stream = torch.cuda.current_stream()
    return C.c_void_p(stream.cuda_stream)


class Context:
    """One sp_ctx.  Methods carry the names of the C entry points."""

    def __init__(self, profile, max_requests: int, device: int = 0, policy=None):
        self.lib = load_library()
        self.profile = profile
        self.device = device
        self.max_requests = int(max_requests)
        st, keep = marshal_profile(profile, max_requests)
        h = C.c_void_p()
        rc = self.lib.sp_create(C.byref(st), device, C.byref(h))
        if rc != SP_OK:
            raise SneakPeekError(rc, "sp_create", self.lib.sp_strerror(rc).decode())
        self.h = h
        self.m_max = self.lib.sp_max_models(h)
        self.c_max = self.lib.sp_max_classes(h)
        self.rounds_in_one_launch = bool(self.lib.sp_rounds_in_one_launch(h))
        self.n = 0
        if policy is not None:
            self.sp_set_policy(policy)
        if getattr(profile, "swap_ms", None) is not None:
            for a in range(int(profile.n_apps)):
                if profile.swap_ms[a] is not None:
                    self.sp_set_swap_cost(a, profile.swap_ms[a])
        if getattr(profile, "prior_alpha", None) is not None:
            for a in range(int(profile.n_apps)):
                if profile.prior_alpha[a] is not None:
                    self.sp_set_prior(a, profile.prior_alpha[a], float(profile.evidence_k[a]))

    def _check(self, rc, where, ok=(SP_OK,)):
        if rc not in ok:
            raise SneakPeekError(rc, where, self.lib.sp_strerror(rc).decode() + " " +
                                 self.lib.sp_last_hip_error(self.h).decode())
        return rc

    def close(self):
        if getattr(self, "h", None):
            self.lib.sp_destroy(self.h)
            self.h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def sp_score(self, x, app, deadline_ms, weight, ea_out=None, key_out=None, stream=None):
        """Tensors live on the context's device; x is float32 or (bf16 bits) int16/uint16/bfloat16."""
        n = int(app.shape[0])
        self.n = n
        rc = self.lib.sp_score(self.h, n, _dptr(x), _dptr(app), _dptr(deadline_ms), _dptr(weight),
                               _stream_ptr(stream), _dptr(ea_out), _dptr(key_out))
        return self._check(rc, "sp_score")

    def sp_greedy_round(self, req_ids_out=None, stream=None):
        """Returns (status, decision dict or None)."""
        d = sp_decision()
        rc = self.lib.sp_greedy_round(self.h, _stream_ptr(stream), C.byref(d), _dptr(req_ids_out))
        self._check(rc, "sp_greedy_round", ok=(SP_OK, SP_DONE))
        return rc, (d.as_dict() if rc == SP_OK else None)

    def sp_greedy_round_static(self, req_ids_out=None, stream=None):
        """sp_greedy_round on the library's static scratch array; returns (status, decision dict or None)."""
        d = sp_decision()
        rc = self.lib.sp_greedy_round_static(self.h, _stream_ptr(stream), C.byref(d), _dptr(req_ids_out))
        self._check(rc, "sp_greedy_round_static", ok=(SP_OK, SP_DONE))
        return rc, (d.as_dict() if rc == SP_OK else None)

    def sp_schedule(self, max_rounds=0, model_out=None, round_out=None, order_out=None, util_out=None,
                    log_capacity=0, stream=None):
        """Returns (status, summary dict, list of decision dicts)."""
        log = (sp_decision * max(1, log_capacity))()
        sm = sp_summary()
        rc = self.lib.sp_schedule(self.h, int(max_rounds), _stream_ptr(stream), _dptr(model_out), _dptr(round_out),
                                  _dptr(order_out), _dptr(util_out), log, int(log_capacity), C.byref(sm))
        self._check(rc, "sp_schedule", ok=(SP_OK, SP_DONE))
        n_log = min(sm.n_rounds, log_capacity)
        return rc, sm.as_dict(), [log[i].as_dict() for i in range(n_log)]

    def sp_set_prior(self, app, alpha, evidence_k):
        """alpha: host array of C_a floats, or None to remove the application's prior."""
        if alpha is None:
            return self._check(self.lib.sp_set_prior(self.h, int(app), None, C.c_float(0.0)), "sp_set_prior")
        buf = np.ascontiguousarray(alpha, dtype=np.float32)
        return self._check(self.lib.sp_set_prior(self.h, int(app), buf.ctypes.data_as(C.c_void_p),
                                                 C.c_float(float(evidence_k))), "sp_set_prior")

    def sp_set_policy(self, policy):
        """policy: an object with the fields of sp_policy (workloads.Policy), or None for the default."""
        if policy is None:
            return self._check(self.lib.sp_set_policy(self.h, None), "sp_set_policy")
        st = sp_policy(int(policy.order), int(policy.select), int(policy.batch_rule), int(policy.choice),
                       int(policy.weight), int(policy.batch_cap), int(getattr(policy, "split_groups", 0)))
        return self._check(self.lib.sp_set_policy(self.h, C.byref(st)), "sp_set_policy")

    def sp_set_swap_cost(self, app, swap_ms):
        """swap_ms: host array of M_a floats, or None for no swap-in cost."""
        if swap_ms is None:
            return self._check(self.lib.sp_set_swap_cost(self.h, int(app), None), "sp_set_swap_cost")
        buf = np.ascontiguousarray(swap_ms, dtype=np.float32)
        return self._check(self.lib.sp_set_swap_cost(self.h, int(app), buf.ctypes.data_as(C.c_void_p)),
                           "sp_set_swap_cost")

    def sp_set_timing(self, level=1):
        """0 off, 1 stage events, 2 stage events and one event per round, 3 events around the scoring kernel only."""
        return self._check(self.lib.sp_set_timing(self.h, int(level)), "sp_set_timing")

    def sp_get_timing(self):
        t = sp_timing()
        self._check(self.lib.sp_get_timing(self.h, C.byref(t)), "sp_get_timing")
        return t.as_dict()

    def sp_get_round_times(self, capacity=4096):
        buf = (C.c_float * capacity)()
        n = C.c_int32(0)
        self._check(self.lib.sp_get_round_times(self.h, buf, capacity, C.byref(n)), "sp_get_round_times")
        return [buf[i] for i in range(n.value)]

    def sp_debug_set_spin_limit(self, polls):
        return self._check(self.lib.sp_debug_set_spin_limit(self.h, int(polls)), "sp_debug_set_spin_limit")

    def sp_debug_set_sort_spin_limit(self, polls):
        return self._check(self.lib.sp_debug_set_sort_spin_limit(self.h, int(polls)), "sp_debug_set_sort_spin_limit")

    def sp_debug_set_generation(self, generation):
        return self._check(self.lib.sp_debug_set_generation(self.h, int(generation)), "sp_debug_set_generation")

    def sp_debug_dump(self, kind, dst, x=None, app=None, stream=None):
        rc = self.lib.sp_debug_dump(self.h, int(kind), _stream_ptr(stream), _dptr(x), _dptr(app), _dptr(dst))
        return self._check(rc, "sp_debug_dump")


def sp_debug_mfma_rate(random_bits: bool, iters: int = 16384, idle: int = 0, device: int = 0, stream=None):
    """(TFLOP/s, shader clock in GHz) of the bare matrix-core loop; see include/sneakpeek.h."""
    lib = load_library()
    tf, ghz = C.c_double(0.0), C.c_double(0.0)
    rc = lib.sp_debug_mfma_rate(int(device), int(bool(random_bits)), int(idle), int(iters), _stream_ptr(stream),
                                C.byref(tf), C.byref(ghz))
    if rc != SP_OK:
        raise SneakPeekError(rc, "sp_debug_mfma_rate")
    return tf.value, ghz.value


def sp_debug_copy_rate(n_bytes: int = 1 << 28, device: int = 0, stream=None):
    """GB/s (read + written) of a plain streaming copy kernel; see include/sneakpeek.h."""
    lib = load_library()
    gbs = C.c_double(0.0)
    rc = lib.sp_debug_copy_rate(int(device), int(n_bytes), _stream_ptr(stream), C.byref(gbs))
    if rc != SP_OK:
        raise SneakPeekError(rc, "sp_debug_copy_rate")
    return gbs.value


def to_device(requests, device="cuda:0"):
    """Upload one window's request arrays; returns (x, app, deadline, weight) tensors."""
    import torch
    x = requests.x
    if x.dtype == np.uint16:
        xt = torch.from_numpy(x.view(np.int16)).to(device)
    else:
        xt = torch.from_numpy(x).to(device)
    return (xt, torch.from_numpy(requests.app).to(device),
            torch.from_numpy(requests.deadline_rel_ms).to(device), torch.from_numpy(requests.weight).to(device))
