"""ctypes binding of include/dblp_agg.h.  Same names, same argument order.

Device buffers are torch CUDA(HIP) tensors; only their data_ptr() crosses the
boundary.  torch is plumbing here (device memory, streams), not compute.
"""
from __future__ import annotations

import ctypes
import os

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
LIB_PATH = os.environ.get("DBLP_AGG_LIB") or os.path.join(_HERE, "libdblp_agg.so")

OK, EINVAL, ENOMEM, ECAPACITY, ESTATE, EHIP = 0, -1, -2, -3, -4, -5
_NAMES = {EINVAL: "DBLP_EINVAL", ENOMEM: "DBLP_ENOMEM", ECAPACITY: "DBLP_ECAPACITY",
          ESTATE: "DBLP_ESTATE", EHIP: "DBLP_EHIP"}
COMP_ZEROFILL_MEAN = 0
K_INDEX, K_GATHER, K_PROBE, K_FINALIZE, K_GATHER_DIRECT = 0, 1, 2, 3, 4
K_COUNT = 5
ACC_AUTO, ACC_FIRST, ACC_SECOND, ACC_ALTERNATE = 0, 1, 2, 3
ACCMODE_SINGLE, ACCMODE_PAIR, ACCMODE_SEARCH = 0, 1, 2

EXPORTS = ["dblp_create", "dblp_destroy", "dblp_layout", "dblp_accumulator_copies", "dblp_accumulator_policy", "dblp_accumulator_info", "dblp_accumulator_ptr", "dblp_begin_round", "dblp_packetize", "dblp_packetize_list",
           "dblp_apply_arrivals", "dblp_apply_arrivals_queue", "dblp_loss_account", "dblp_finalize", "dblp_phase_signal",
           "dblp_get_bitmap", "dblp_get_counters", "dblp_set_prev_norm", "dblp_get_prev_norm",
           "dblp_last_error", "dblp_profile_enable", "dblp_profile_read", "dblp_policy_two_level", "dblp_policy_three_level", "dblp_policy_linear", "dblp_clr_init", "dblp_clr_step",
           "dblp_sumsq_static", "dblp_sumsq_static_error"]


class DblpError(RuntimeError):
    def __init__(self, code: int, msg: str):
        super().__init__(f"{_NAMES.get(code, code)}: {msg}")
        self.code = code


class _Bucket(ctypes.Structure):
    _fields_ = [("elem_offset", ctypes.c_uint64), ("elem_count", ctypes.c_uint64)]


class ClrState(ctypes.Structure):
    """dblp_clr_state: the caller-owned state of the epoch-level tolerance controller."""
    _fields_ = [("p_low_ppm", ctypes.c_uint32), ("p_high_ppm", ctypes.c_uint32),
                ("iters_per_epoch", ctypes.c_uint32), ("bound_ppm", ctypes.c_uint32),
                ("step", ctypes.c_uint64)]


class _Config(ctypes.Structure):
    _fields_ = [("n_workers", ctypes.c_uint32), ("payload_floats", ctypes.c_uint32),
                ("n_elems", ctypes.c_uint64), ("n_buckets", ctypes.c_uint32),
                ("buckets", ctypes.POINTER(_Bucket)), ("eta", ctypes.c_double),
                ("device", ctypes.c_int), ("stream", ctypes.c_void_p),
                ("accumulator_mode", ctypes.c_int), ("d_accumulator", ctypes.c_void_p * 2),
                ("search_free_fraction", ctypes.c_double), ("search_seconds", ctypes.c_double)]


_lib = None


def lib():
    """Loads the built library; raises if it is missing (there is no fallback path)."""
    global _lib
    if _lib is None:
        if not os.path.exists(LIB_PATH):
            raise RuntimeError(f"{LIB_PATH} is not built: run `python -c 'import __graft_entry__ as g; g.build()'`")
        L = ctypes.CDLL(LIB_PATH)
        vp, u64, u32, u16, i32, dbl = (ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32,
                                       ctypes.c_uint16, ctypes.c_int, ctypes.c_double)
        L.dblp_create.argtypes = [ctypes.POINTER(vp), ctypes.POINTER(_Config)]
        L.dblp_destroy.argtypes = [vp]
        L.dblp_layout.argtypes = [vp, ctypes.POINTER(u64), ctypes.POINTER(u32), ctypes.POINTER(u64)]
        L.dblp_begin_round.argtypes = [vp, u16]
        L.dblp_accumulator_copies.argtypes = [vp, i32, i32]
        L.dblp_accumulator_policy.argtypes = [vp, i32]
        L.dblp_accumulator_info.argtypes = [vp, ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(i32), ctypes.POINTER(dbl)]
        L.dblp_accumulator_ptr.argtypes = [vp, i32, ctypes.POINTER(vp)]
        L.dblp_packetize.argtypes = [vp, u32, u16, vp, u64, u64, u64, u64, vp, u64, u64, vp, vp]
        L.dblp_packetize_list.argtypes = [vp, u16, ctypes.POINTER(vp), vp, u64, u64, u64, vp, vp]
        L.dblp_apply_arrivals.argtypes = [vp, vp, vp, u64, vp, vp, u64]
        L.dblp_apply_arrivals_queue.argtypes = [vp, vp, u64, vp, u64]
        L.dblp_loss_account.argtypes = [vp, u32, vp, vp, u64, ctypes.POINTER(u64), ctypes.POINTER(i32)]
        L.dblp_finalize.argtypes = [vp, i32, vp]
        L.dblp_phase_signal.argtypes = [vp, vp, ctypes.POINTER(dbl), ctypes.POINTER(dbl), ctypes.POINTER(i32)]
        L.dblp_get_bitmap.argtypes = [vp, vp]
        L.dblp_get_counters.argtypes = [vp, ctypes.POINTER(u64)]
        L.dblp_set_prev_norm.argtypes = [vp, dbl, i32]
        L.dblp_get_prev_norm.argtypes = [vp, ctypes.POINTER(dbl), ctypes.POINTER(i32)]
        L.dblp_profile_enable.argtypes = [vp, i32]
        L.dblp_profile_read.argtypes = [vp, i32, ctypes.POINTER(dbl), ctypes.POINTER(u64)]
        L.dblp_last_error.argtypes = [vp]
        L.dblp_last_error.restype = ctypes.c_char_p
        for name in ("dblp_policy_two_level", "dblp_policy_three_level", "dblp_policy_linear"):
            getattr(L, name).restype = u32
        L.dblp_clr_init.argtypes = [ctypes.POINTER(ClrState), u32, u32, u32]
        L.dblp_clr_step.argtypes = [ctypes.POINTER(ClrState), i32]
        L.dblp_clr_step.restype = u32
        L.dblp_sumsq_static.argtypes = [i32, vp, vp, u64, vp]
        L.dblp_sumsq_static_error.restype = ctypes.c_char_p
        L.dblp_policy_two_level.argtypes = [i32, u32, u32]
        L.dblp_policy_three_level.argtypes = [dbl, dbl, u32, u32, u32]
        L.dblp_policy_linear.argtypes = [dbl, dbl, u32, u32]
        _lib = L
    return _lib


def policy_two_level(critical: bool, p_low_ppm: int, p_high_ppm: int) -> int:
    return int(lib().dblp_policy_two_level(int(critical), p_low_ppm, p_high_ppm))


def policy_three_level(rel_delta: float, eta: float, tight_ppm: int, mid_ppm: int, loose_ppm: int) -> int:
    return int(lib().dblp_policy_three_level(rel_delta, eta, tight_ppm, mid_ppm, loose_ppm))


def policy_linear(rel_delta: float, eta: float, lo_ppm: int, hi_ppm: int) -> int:
    return int(lib().dblp_policy_linear(rel_delta, eta, lo_ppm, hi_ppm))


def sumsq_static(d_vec, d_sumsq, n_elems=None, device=0, stream=None):
    """dblp_sumsq_static: sum of squares of a device vector into a device double, allocating nothing."""
    import torch
    if stream is None:
        stream = torch.cuda.current_stream(device).cuda_stream
    rc = lib().dblp_sumsq_static(device, stream, _ptr(d_vec), d_vec.numel() if n_elems is None else n_elems, _ptr(d_sumsq))
    if rc != OK:
        raise DblpError(rc, lib().dblp_sumsq_static_error().decode())


class ClrController:
    """Epoch-level tolerance controller (dblp_clr_init / dblp_clr_step)."""

    def __init__(self, p_low_ppm: int, p_high_ppm: int, iters_per_epoch: int):
        self.state = ClrState()
        rc = lib().dblp_clr_init(ctypes.byref(self.state), p_low_ppm, p_high_ppm, iters_per_epoch)
        if rc != OK:
            raise DblpError(rc, "dblp_clr_init: bad arguments")

    @property
    def bound_ppm(self) -> int:
        return int(self.state.bound_ppm)

    def step(self, critical: bool) -> int:
        return int(lib().dblp_clr_step(ctypes.byref(self.state), int(critical)))


def _ptr(t):
    return None if t is None else t.data_ptr()


class Aggregator:
    """One dblp_ctx.  Methods mirror the C entry points one to one."""

    def __init__(self, n_workers, n_elems, payload_floats, bucket_off, bucket_cnt, eta=0.5, device=0, stream=None,
                 accumulator_mode=ACCMODE_SINGLE, d_accumulator=(None, None), search_free_fraction=0.0,
                 search_seconds=0.0):
        """d_accumulator: up to two caller-owned device tensors of n_elems floats (kept alive here)."""
        import torch
        off = np.asarray(bucket_off, dtype=np.uint64)
        cnt = np.asarray(bucket_cnt, dtype=np.uint64)
        arr = (_Bucket * off.size)(*[_Bucket(int(o), int(c)) for o, c in zip(off, cnt)])
        if stream is None:
            stream = torch.cuda.current_stream(device).cuda_stream
        self._caller_acc = tuple(d_accumulator)
        acc = (ctypes.c_void_p * 2)(*[_ptr(t) for t in self._caller_acc])
        cfg = _Config(n_workers, payload_floats, n_elems, off.size, arr, eta, device, stream,
                      accumulator_mode, acc, search_free_fraction, search_seconds)
        h = ctypes.c_void_p()
        rc = lib().dblp_create(ctypes.byref(h), ctypes.byref(cfg))
        if rc != OK:
            raise DblpError(rc, "dblp_create failed")
        self._h = h
        self.W, self.N, self.P, self.B = int(n_workers), int(n_elems), int(payload_floats), int(off.size)
        self.device = torch.device("cuda", device)
        n, s, wpw = ctypes.c_uint64(), ctypes.c_uint32(), ctypes.c_uint64()
        self._check(lib().dblp_layout(self._h, ctypes.byref(n), ctypes.byref(s), ctypes.byref(wpw)))
        self.n_pkts, self.stride, self.words_pw = int(n.value), int(s.value), int(wpw.value)

    def _check(self, rc, allow=()):
        if rc != OK and rc not in allow:
            raise DblpError(rc, lib().dblp_last_error(self._h).decode())
        return rc

    def close(self):
        if getattr(self, "_h", None):
            lib().dblp_destroy(self._h)
            self._h = None

    def __del__(self):
        try:
            self.close()
        except Exception:
            pass

    def begin_round(self, rnd: int):
        self._check(lib().dblp_begin_round(self._h, rnd & 0xFFFF))

    def packetize(self, w, rnd, d_grad, elem_base, first_seq, n_pkts, d_packets, d_src_worker,
                  d_slot_map=None, slot_base=0, n_slots=None):
        if n_slots is None:
            n_slots = d_src_worker.numel()
        self._check(lib().dblp_packetize(self._h, w, rnd & 0xFFFF, _ptr(d_grad), elem_base, d_grad.numel(),
                                         first_seq, n_pkts, _ptr(d_slot_map), slot_base, n_slots,
                                         _ptr(d_packets), _ptr(d_src_worker)))

    def packetize_list(self, rnd, d_grads, d_retx_list, n_entries, d_packets, d_src_worker, slot_base=0, n_slots=None):
        """d_grads: one device tensor per worker (whole gradient)."""
        if n_slots is None:
            n_slots = d_src_worker.numel()
        ptrs = (ctypes.c_void_p * self.W)(*[t.data_ptr() for t in d_grads])
        self._check(lib().dblp_packetize_list(self._h, rnd & 0xFFFF, ptrs, _ptr(d_retx_list), n_entries, slot_base,
                                              n_slots, _ptr(d_packets), _ptr(d_src_worker)))

    def accumulator_copies(self, copies: int, place: int = 0):
        """place: 0 plain second allocation, 1 bounded search for one in another third of HBM."""
        self._check(lib().dblp_accumulator_copies(self._h, copies, int(place)))

    def accumulator_ptr(self, which: int = 0) -> int:
        p = ctypes.c_void_p()
        self._check(lib().dblp_accumulator_ptr(self._h, which, ctypes.byref(p)))
        return int(p.value)

    def accumulator_tensor(self, which: int = 0):
        """A torch view (no copy) of accumulator copy `which`: after an in-place finalize, copy 0 is
        the aggregated gradient.  Valid while the context lives and its copies are not reallocated."""
        import torch

        class _View:
            __cuda_array_interface__ = dict(shape=(self.N,), typestr="<f4", data=(self.accumulator_ptr(which), False),
                                            version=2, strides=None)
        return torch.as_tensor(_View(), device=self.device)

    def accumulator_policy(self, policy: int):
        self._check(lib().dblp_accumulator_policy(self._h, policy))

    def accumulator_info(self) -> dict:
        n, d, p, ms = ctypes.c_int(), ctypes.c_int(), ctypes.c_int(), (ctypes.c_double * 4)()
        self._check(lib().dblp_accumulator_info(self._h, ctypes.byref(n), ctypes.byref(d), ctypes.byref(p), ms))
        return dict(copies=n.value, distinct_thirds=bool(d.value), last_pick=p.value,
                    placement_ms=[round(ms[0], 4), round(ms[1], 4)], placement_steps=int(ms[2]),
                    placement_seconds=round(ms[3], 3))

    def apply_arrivals(self, d_packets, d_src_worker, n_slots, d_mask_words=None, d_order=None, n_arrivals=None):
        if n_arrivals is None:
            n_arrivals = d_order.numel() if d_order is not None else n_slots
        self._check(lib().dblp_apply_arrivals(self._h, _ptr(d_packets), _ptr(d_src_worker), n_slots,
                                              _ptr(d_mask_words), _ptr(d_order), n_arrivals))

    def apply_arrivals_queue(self, d_packets, n_slots, d_queue, n_arrivals=None):
        if n_arrivals is None:
            n_arrivals = d_queue.numel()
        self._check(lib().dblp_apply_arrivals_queue(self._h, _ptr(d_packets), n_slots, _ptr(d_queue), n_arrivals))

    def loss_account(self, bound_ppm, d_missing, d_retx_list, capacity=None):
        """Returns (count, all_met, truncated)."""
        cap = (0 if d_retx_list is None else d_retx_list.numel()) if capacity is None else capacity
        count, met = ctypes.c_uint64(), ctypes.c_int()
        rc = self._check(lib().dblp_loss_account(self._h, bound_ppm, _ptr(d_missing), _ptr(d_retx_list), cap,
                                                 ctypes.byref(count), ctypes.byref(met)), allow=(ECAPACITY,))
        return int(count.value), bool(met.value), rc == ECAPACITY

    def finalize(self, d_out=None, compensation=COMP_ZEROFILL_MEAN):
        """d_out None: in place (the result is accumulator copy 0)."""
        self._check(lib().dblp_finalize(self._h, compensation, _ptr(d_out)))

    def phase_signal(self, d_vec=None):
        norm, delta, crit = ctypes.c_double(), ctypes.c_double(), ctypes.c_int()
        self._check(lib().dblp_phase_signal(self._h, _ptr(d_vec), ctypes.byref(norm), ctypes.byref(delta),
                                            ctypes.byref(crit)))
        return norm.value, delta.value, bool(crit.value)

    def get_bitmap(self, d_bitmap_out):
        self._check(lib().dblp_get_bitmap(self._h, _ptr(d_bitmap_out)))

    def get_counters(self) -> dict:
        c = (ctypes.c_uint64 * 4)()
        self._check(lib().dblp_get_counters(self._h, c))
        return dict(accepted=int(c[0]), duplicate=int(c[1]), stale=int(c[2]), invalid=int(c[3]))

    def profile_enable(self, on):
        """on: False/0 off, True all kernel groups, or a bit mask (1 << K_GATHER, ...)."""
        self._check(lib().dblp_profile_enable(self._h, (1 << K_COUNT) - 1 if on is True else int(on)))

    def profile_read(self, kernel: int):
        """(total milliseconds, launches) of one kernel group since the last read."""
        ms, n = ctypes.c_double(), ctypes.c_uint64()
        self._check(lib().dblp_profile_read(self._h, kernel, ctypes.byref(ms), ctypes.byref(n)))
        return ms.value, int(n.value)

    def set_prev_norm(self, norm):
        self._check(lib().dblp_set_prev_norm(self._h, 0.0 if norm is None else norm, int(norm is not None)))

    def get_prev_norm(self):
        v, have = ctypes.c_double(), ctypes.c_int()
        self._check(lib().dblp_get_prev_norm(self._h, ctypes.byref(v), ctypes.byref(have)))
        return v.value if have.value else None
