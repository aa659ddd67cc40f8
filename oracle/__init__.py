"""ctypes front end of the CPU oracle (oracle/dblp_oracle.c).

TEST INFRASTRUCTURE ONLY: imported by tests/, by __graft_entry__.smoke() and by
the cpu_baseline leg of bench.py.  Nothing in the product package may import it.
All arrays are numpy host arrays.
"""
from __future__ import annotations

import ctypes
import os
import subprocess

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
_lib = None


def build(force: bool = False) -> str:
    so = os.path.join(_HERE, "libdblp_oracle.so")
    src = os.path.join(_HERE, "dblp_oracle.c")
    if force or not os.path.exists(so) or os.path.getmtime(so) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-std=c11", "-fopenmp", "-Wall", "-Wextra", "-shared", "-fPIC",
                               "-o", so, src, "-lm"])
    return so


def lib():
    global _lib
    if _lib is None:
        L = ctypes.CDLL(build())
        vp, u64, u32, u16, i32, dbl = (ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint32,
                                       ctypes.c_uint16, ctypes.c_int, ctypes.c_double)
        L.oracle_create.restype = vp
        L.oracle_create.argtypes = [u32, u64, u32, u32, vp, vp, dbl]
        L.oracle_destroy.argtypes = [vp]
        L.oracle_n_pkts.restype = u64
        L.oracle_n_pkts.argtypes = [vp]
        L.oracle_begin_round.argtypes = [vp, u16]
        L.oracle_packetize.restype = i32
        L.oracle_packetize.argtypes = [vp, u32, u16, vp, u64, u64, u64, u64, vp, u64, vp, u64, vp]
        L.oracle_write_headers.restype = i32
        L.oracle_write_headers.argtypes = [vp, u32, u16, u64, u64, vp, u64, vp, vp]
        L.oracle_apply_arrivals.argtypes = [vp, vp, u64, vp, u64, vp, vp, u64, i32]
        L.oracle_apply_arrivals_mt.restype = i32
        L.oracle_apply_arrivals_mt.argtypes = [vp, vp, u64, vp, u64, vp, vp, u64, i32, i32]
        L.oracle_loss_account.argtypes = [vp, u32, vp, vp, u64, vp, vp]
        L.oracle_finalize.argtypes = [vp, vp]
        L.oracle_phase_signal.argtypes = [vp, vp, vp, vp, vp]
        L.oracle_set_prev_norm.argtypes = [vp, dbl, i32]
        L.oracle_get_received.argtypes = [vp, vp]
        L.oracle_get_acc.argtypes = [vp, vp]
        L.oracle_get_counters.argtypes = [vp, vp]
        L.oracle_policy_two_level.restype = u32
        L.oracle_policy_two_level.argtypes = [i32, u32, u32]
        L.oracle_policy_three_level.restype = u32
        L.oracle_policy_three_level.argtypes = [dbl, dbl, u32, u32, u32]
        L.oracle_policy_linear.restype = u32
        L.oracle_policy_linear.argtypes = [dbl, dbl, u32, u32]
        L.oracle_clr_trace.argtypes = [u32, u32, u32, vp, u64, vp]
        _lib = L
    return _lib


def _p(a):
    return None if a is None else a.ctypes.data


class Oracle:
    """One receiver: W workers, N elements, P payload floats, buckets tiling [0, N)."""

    def __init__(self, W, N, P, bucket_off, bucket_cnt, eta=0.5):
        off = np.ascontiguousarray(bucket_off, dtype=np.uint64)
        cnt = np.ascontiguousarray(bucket_cnt, dtype=np.uint64)
        self.W, self.N, self.P, self.B = int(W), int(N), int(P), int(off.size)
        self._h = lib().oracle_create(self.W, self.N, self.P, self.B, _p(off), _p(cnt), float(eta))
        if not self._h:
            raise ValueError("oracle_create rejected the configuration")
        self.n_pkts = int(lib().oracle_n_pkts(self._h))
        self.stride = (8 + 4 * self.P + 15) // 16 * 16
        self._prev = None      # the stored previous norm, as last set or computed (for reporting only)

    def close(self):
        if self._h:
            lib().oracle_destroy(self._h)
            self._h = None

    def __del__(self):
        self.close()

    def begin_round(self, rnd: int):
        lib().oracle_begin_round(self._h, rnd & 0xFFFF)

    def packetize(self, w, rnd, grad, elem_base, first_seq, n, packets, src_worker, slot_map=None, slot_base=0):
        grad = np.ascontiguousarray(grad, dtype=np.float32)
        assert packets.dtype == np.uint8 and src_worker.dtype == np.uint16
        if slot_map is not None:
            slot_map = np.ascontiguousarray(slot_map, dtype=np.uint32)
            assert slot_map.size == n
        rc = lib().oracle_packetize(self._h, w, rnd & 0xFFFF, _p(grad), elem_base, grad.size, first_seq, n,
                                    _p(slot_map), slot_base, _p(packets), self.stride, _p(src_worker))
        if rc != 0:
            raise ValueError("oracle_packetize: packet outside the gradient window")

    def write_headers(self, w, rnd, first_seq, n, headers, src_worker, slot_map=None, slot_base=0):
        """The 8 header bytes of packets first_seq .. first_seq + n - 1 of worker w, one per slot of
        `headers` (uint8, 8 bytes per slot): the input of apply_arrivals(accumulate=False, stride=8)."""
        assert headers.dtype == np.uint8 and src_worker.dtype == np.uint16
        if slot_map is not None:
            slot_map = np.ascontiguousarray(slot_map, dtype=np.uint32)
            assert slot_map.size == n
        rc = lib().oracle_write_headers(self._h, w, rnd & 0xFFFF, first_seq, n, _p(slot_map), slot_base,
                                        _p(headers), _p(src_worker))
        if rc != 0:
            raise ValueError("oracle_write_headers: sequence number out of range")

    def apply_arrivals(self, packets, src_worker, n_slots, mask=None, order=None, n_arrivals=None,
                       accumulate=True, stride=None, threads=None):
        """threads: None = the plain single-threaded walk; an integer = the element-range-parallel
        walk on that many threads (0: all that OpenMP offers); returns the number used."""
        if mask is not None:
            mask = np.ascontiguousarray(mask, dtype=np.uint64)
            assert mask.size * 64 >= n_slots
        if order is not None:
            order = np.ascontiguousarray(order, dtype=np.uint32)
            if n_arrivals is None:
                n_arrivals = order.size
            assert order.size >= n_arrivals
        elif n_arrivals is None:
            n_arrivals = n_slots
        if threads is not None:
            return int(lib().oracle_apply_arrivals_mt(self._h, _p(packets), stride or self.stride, _p(src_worker),
                                                      n_slots, _p(mask), _p(order), n_arrivals, int(accumulate),
                                                      int(threads)))
        lib().oracle_apply_arrivals(self._h, _p(packets), stride or self.stride, _p(src_worker), n_slots,
                                    _p(mask), _p(order), n_arrivals, int(accumulate))
        return 1

    def loss_account(self, bound_ppm: int, capacity: int | None = None):
        cap = self.W * self.n_pkts if capacity is None else capacity
        missing = np.empty(self.W * self.B, dtype=np.uint32)
        lst = np.empty(max(cap, 1), dtype=np.uint64)
        count = ctypes.c_uint64()
        met = ctypes.c_int()
        lib().oracle_loss_account(self._h, bound_ppm, _p(missing), _p(lst), cap, ctypes.byref(count),
                                  ctypes.byref(met))
        return missing.reshape(self.W, self.B), lst[:min(count.value, cap)].copy(), int(count.value), bool(met.value)

    def finalize(self) -> np.ndarray:
        out = np.empty(self.N, dtype=np.float64)
        lib().oracle_finalize(self._h, _p(out))
        return out

    def phase_signal(self, out: np.ndarray):
        out = np.ascontiguousarray(out, dtype=np.float64)
        assert out.size == self.N
        norm, delta, crit = ctypes.c_double(), ctypes.c_double(), ctypes.c_int()
        lib().oracle_phase_signal(self._h, _p(out), ctypes.byref(norm), ctypes.byref(delta), ctypes.byref(crit))
        self._prev = norm.value
        return norm.value, delta.value, bool(crit.value)

    def set_prev_norm(self, v: float | None):
        lib().oracle_set_prev_norm(self._h, 0.0 if v is None else float(v), int(v is not None))
        self._prev = v

    def get_prev_norm(self):
        return self._prev

    def received(self) -> np.ndarray:
        out = np.empty((self.W, self.n_pkts), dtype=np.uint8)
        lib().oracle_get_received(self._h, _p(out))
        return out

    def acc(self) -> np.ndarray:
        out = np.empty(self.N, dtype=np.float64)
        lib().oracle_get_acc(self._h, _p(out))
        return out

    def counters(self) -> dict:
        c = np.zeros(4, dtype=np.uint64)
        lib().oracle_get_counters(self._h, _p(c))
        return dict(accepted=int(c[0]), duplicate=int(c[1]), stale=int(c[2]), invalid=int(c[3]))


def policy_two_level(critical: bool, p_low_ppm: int, p_high_ppm: int) -> int:
    return int(lib().oracle_policy_two_level(int(critical), p_low_ppm, p_high_ppm))


def policy_three_level(rel_delta: float, eta: float, tight_ppm: int, mid_ppm: int, loose_ppm: int) -> int:
    return int(lib().oracle_policy_three_level(rel_delta, eta, tight_ppm, mid_ppm, loose_ppm))


def policy_linear(rel_delta: float, eta: float, lo_ppm: int, hi_ppm: int) -> int:
    return int(lib().oracle_policy_linear(rel_delta, eta, lo_ppm, hi_ppm))


def clr_trace(p_low_ppm: int, p_high_ppm: int, iters_per_epoch: int, critical) -> np.ndarray:
    """Threshold in force after each step of the epoch-level controller."""
    crit = np.ascontiguousarray(critical, dtype=np.uint8)
    out = np.empty(crit.size, dtype=np.uint32)
    lib().oracle_clr_trace(p_low_ppm, p_high_ppm, iters_per_epoch, _p(crit), crit.size, _p(out))
    return out
