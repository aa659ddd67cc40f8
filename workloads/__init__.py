"""Seeded synthetic inputs for bounded-loss gradient aggregation.

Everything here manufactures INPUTS only: bucket tables, gradient values,
packet-survival patterns, wire placement and arrival orders.  None of the
protocol's arithmetic (packet parsing, accumulation, loss accounting,
compensation, norm) lives in this package; the CPU checker and the GPU library
both consume its outputs and share nothing else.

The shapes mirror the workloads listed for the DBLP receiver path: a flat
1M-element gradient cut into 256-float packets, ResNet-50- and GPT-2-sized
per-tensor bucket tables with 366-float (MTU-filling) packets, and a 1.3B
gradient streamed in 256 MB chunks.  The paper's real gradients need its
datasets and training runs; these stand in for them.
"""
from __future__ import annotations

import ctypes
import os
import subprocess
from dataclasses import dataclass, field

import numpy as np

_HERE = os.path.dirname(os.path.abspath(__file__))
MASTER_SEED = 0x260501989

STREAM_GRAD, STREAM_LOSS, STREAM_ORDER, STREAM_BUCKETS, STREAM_PLACE, STREAM_WINDOWS = 1, 2, 3, 4, 5, 6

_GOLDEN = np.uint64(0x9E3779B97F4A7C15)
_TAILSALT = np.uint64(0xD1B54A32D192ED03)


# ----------------------------------------------------------------------------
# native generator libraries
# ----------------------------------------------------------------------------
def build_cpu(force: bool = False) -> str:
    so = os.path.join(_HERE, "libdblp_gen.so")
    src = os.path.join(_HERE, "gen.c")
    if force or not os.path.exists(so) or os.path.getmtime(so) < os.path.getmtime(src):
        subprocess.check_call(["gcc", "-O2", "-fopenmp", "-shared", "-fPIC", "-o", so, src])
    return so


def build_hip() -> str:
    so = os.path.join(_HERE, "libdblp_gen_hip.so")
    src = os.path.join(_HERE, "gen.hip")
    subprocess.check_call(
        ["/opt/rocm/bin/hipcc", "--offload-arch=gfx950", "-O3", "-shared", "-fPIC",
         "-Xclang", "-target-feature", "-Xclang", "-packed-fp32-ops", "-o", so, src])
    return so


_cpu = None
_hip = None


def _cpu_lib():
    global _cpu
    if _cpu is None:
        lib = ctypes.CDLL(build_cpu())
        lib.dblp_gen_key.restype = ctypes.c_uint64
        lib.dblp_gen_key.argtypes = [ctypes.c_uint64] * 3
        lib.dblp_gen_grad_fill.restype = None
        lib.dblp_gen_grad_fill.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64,
                                           ctypes.c_uint64, ctypes.c_float, ctypes.c_uint32,
                                           ctypes.c_float]
        lib.dblp_gen_bernoulli.restype = None
        lib.dblp_gen_bernoulli.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64,
                                           ctypes.c_uint32]
        lib.dblp_gen_gilbert_elliott.restype = None
        lib.dblp_gen_gilbert_elliott.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64,
                                                 ctypes.c_uint32, ctypes.c_uint32, ctypes.c_uint32,
                                                 ctypes.c_uint32]
        _cpu = lib
    return _cpu


def _hip_lib():
    global _hip
    if _hip is None:
        so = os.path.join(_HERE, "libdblp_gen_hip.so")
        if not os.path.exists(so):
            raise RuntimeError("workloads/libdblp_gen_hip.so is not built; run __graft_entry__.build()")
        lib = ctypes.CDLL(so)
        lib.dblp_gen_hip_grad_fill.restype = ctypes.c_int
        lib.dblp_gen_hip_grad_fill.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_uint64,
                                               ctypes.c_uint64, ctypes.c_float, ctypes.c_uint32,
                                               ctypes.c_float, ctypes.c_void_p]
        lib.dblp_gen_hip_resend_slots.restype = ctypes.c_int
        lib.dblp_gen_hip_resend_slots.argtypes = [ctypes.c_void_p, ctypes.c_uint64, ctypes.c_void_p,
                                                  ctypes.c_uint64, ctypes.c_void_p, ctypes.c_void_p]
        _hip = lib
    return _hip


def key(seed: int, stream: int, it: int = 0, rnd: int = 0, w: int = 0) -> int:
    """Per-purpose sub-key: one keyed hash stream per (purpose, iteration, round, worker)."""
    sub = ((it * 64 + rnd) << 16) | w
    return int(_cpu_lib().dblp_gen_key(seed & (2**64 - 1), stream, sub))


def q32(p: float) -> int:
    """Probability -> 32-bit integer threshold (draw < q32 happens with probability p)."""
    return min(int(round(p * 2.0**32)), 2**32 - 1)


# ----------------------------------------------------------------------------
# gradient values
# ----------------------------------------------------------------------------
def grad_scale(sigma: float) -> np.float32:
    return np.float32(sigma / 131072.0)


def grad_values(seed: int, w: int, it: int, e0: int, n: int, sigma: float,
                tail_ppm: int = 0, tail_mul: float = 1.0, out: np.ndarray | None = None) -> np.ndarray:
    """Elements [e0, e0+n) of worker w's gradient at iteration `it` (CPU generator)."""
    if out is None:
        out = np.empty(n, dtype=np.float32)
    assert out.dtype == np.float32 and out.size == n and out.flags.c_contiguous
    _cpu_lib().dblp_gen_grad_fill(out.ctypes.data, e0, n, key(seed, STREAM_GRAD, it, 0, w),
                                  float(grad_scale(sigma)), tail_ppm, tail_mul)
    return out


def grad_fill_device(d_ptr: int, seed: int, w: int, it: int, e0: int, n: int, sigma: float,
                     tail_ppm: int = 0, tail_mul: float = 1.0, stream: int = 0) -> None:
    """Same values as grad_values(), written by the device generator to device memory."""
    rc = _hip_lib().dblp_gen_hip_grad_fill(d_ptr, e0, n, key(seed, STREAM_GRAD, it, 0, w),
                                           float(grad_scale(sigma)), tail_ppm, tail_mul, stream)
    if rc != 0:
        raise RuntimeError(f"device generator launch failed: hipError {rc}")


def resend_slots_device(d_list_ptr: int, n: int, d_slot_of_ptr: int, n_pkts: int, d_out_ptr: int, stream: int = 0) -> None:
    """The simulated sender on the device: out[i] = slot_of[worker_i * n_pkts + seq_i] for the first n
    entries (worker << 32 | seq) of a retransmit list.  All arguments are device addresses."""
    rc = _hip_lib().dblp_gen_hip_resend_slots(d_list_ptr, n, d_slot_of_ptr, n_pkts, d_out_ptr, stream)
    if rc != 0:
        raise RuntimeError(f"device generator launch failed: hipError {rc}")


def _mix64_np(x: np.ndarray) -> np.ndarray:
    x = x.copy()
    x ^= x >> np.uint64(30); x *= np.uint64(0xBF58476D1CE4E5B9)
    x ^= x >> np.uint64(27); x *= np.uint64(0x94D049BB133111EB)
    x ^= x >> np.uint64(31)
    return x


def grad_values_numpy(seed: int, w: int, it: int, e0: int, n: int, sigma: float,
                      tail_ppm: int = 0, tail_mul: float = 1.0) -> np.ndarray:
    """Slow numpy restatement of the recipe, used to cross-check the C and HIP generators."""
    k = np.uint64(key(seed, STREAM_GRAD, it, 0, w))
    e = np.arange(e0, e0 + n, dtype=np.uint64)
    with np.errstate(over="ignore"):
        s = np.zeros(n, dtype=np.int64)
        for j in range(3):
            h = _mix64_np(k + (np.uint64(3) * e + np.uint64(j)) * _GOLDEN)
            s += h.view(np.uint16).reshape(n, 4).astype(np.int64).sum(axis=1)
        z = (2 * s - 12 * 65535).astype(np.int32)
        v = z.astype(np.float32) * grad_scale(sigma)
        if tail_ppm:
            t = _mix64_np((k ^ _TAILSALT) + e * _GOLDEN) >> np.uint64(32)
            sel = ((t * np.uint64(1000000)) >> np.uint64(32)) < np.uint64(tail_ppm)
            v = np.where(sel, v * np.float32(tail_mul), v).astype(np.float32)
    return v


# ----------------------------------------------------------------------------
# geometry: buckets and packets
# ----------------------------------------------------------------------------
@dataclass
class Layout:
    """W workers, N elements, P payload floats per packet, buckets tiling [0, N)."""
    W: int
    N: int
    P: int
    bucket_off: np.ndarray  # uint64[B]
    bucket_cnt: np.ndarray  # uint64[B]
    n_b: np.ndarray = field(init=False)        # packets per bucket
    first_seq: np.ndarray = field(init=False)  # uint64[B+1]

    def __post_init__(self):
        self.bucket_off = np.ascontiguousarray(self.bucket_off, dtype=np.uint64)
        self.bucket_cnt = np.ascontiguousarray(self.bucket_cnt, dtype=np.uint64)
        self.n_b = (self.bucket_cnt + np.uint64(self.P - 1)) // np.uint64(self.P)
        self.first_seq = np.concatenate([[0], np.cumsum(self.n_b)]).astype(np.uint64)

    @property
    def B(self) -> int:
        return int(self.bucket_off.size)

    @property
    def n_pkts(self) -> int:
        return int(self.first_seq[-1])

    @property
    def stride(self) -> int:
        """Wire packet stride: 8-byte header + 4P payload bytes, padded to 16 bytes."""
        return (8 + 4 * self.P + 15) // 16 * 16

    def seq_to_bucket(self, seq: np.ndarray) -> np.ndarray:
        return np.searchsorted(self.first_seq, np.asarray(seq, dtype=np.uint64), side="right") - 1


def buckets_fixed(N: int, P: int, pkts_per_bucket: int):
    per = P * pkts_per_bucket
    off = np.arange(0, N, per, dtype=np.uint64)
    cnt = np.minimum(np.uint64(per), np.uint64(N) - off)
    return off, cnt


def buckets_from_sizes(sizes):
    cnt = np.asarray(sizes, dtype=np.uint64)
    off = np.concatenate([[0], np.cumsum(cnt)[:-1]]).astype(np.uint64)
    return off, cnt


def sizes_loguniform(N: int, B: int, lo: int, hi: int, seed: int) -> np.ndarray:
    """B sizes drawn log-uniform on [lo, hi], scaled to sum to N, rounded, last one fixed up."""
    rng = np.random.Generator(np.random.PCG64(key(seed, STREAM_BUCKETS)))
    raw = np.exp(rng.uniform(np.log(lo), np.log(hi), size=B))
    sizes = np.maximum(1, np.floor(raw * (N / raw.sum()))).astype(np.int64)
    sizes[-1] += N - sizes.sum()
    assert sizes.min() >= 1 and sizes.sum() == N
    return sizes


def sizes_gpt2(d_model: int, n_layer: int, vocab: int = 50257, n_ctx: int = 1024) -> np.ndarray:
    """Parameter-tensor sizes of a GPT-2-style decoder, derived from its hyper-parameters:
    token and position embeddings, then per block {ln, qkv, proj, ln, fc, proj} weight+bias,
    then the final layer norm."""
    d = d_model
    blk = [d, d, d * 3 * d, 3 * d, d * d, d, d, d, d * 4 * d, 4 * d, 4 * d * d, d]
    return np.asarray([vocab * d, n_ctx * d] + blk * n_layer + [d, d], dtype=np.int64)


# ----------------------------------------------------------------------------
# loss patterns (survival bits in (worker, seq) space) -- inputs, seeded
# ----------------------------------------------------------------------------
def survive_bernoulli(seed, it, rnd, W, n_pkts, p) -> np.ndarray:
    out = np.empty((W, n_pkts), dtype=np.uint8)
    for w in range(W):
        _cpu_lib().dblp_gen_bernoulli(out[w].ctypes.data, n_pkts, key(seed, STREAM_LOSS, it, rnd, w), q32(p))
    return out


def survive_gilbert_elliott(seed, it, rnd, W, n_pkts, p_good, p_bad, p_g2b, p_b2g) -> np.ndarray:
    """Per-worker two-state chain over that worker's send sequence (seq order)."""
    out = np.empty((W, n_pkts), dtype=np.uint8)
    lib = _cpu_lib()

    def one(w):   # the chain is sequential per worker; workers are independent (ctypes drops the GIL)
        lib.dblp_gen_gilbert_elliott(out[w].ctypes.data, n_pkts, key(seed, STREAM_LOSS, it, rnd, w),
                                     q32(p_good), q32(p_bad), q32(p_g2b), q32(p_b2g))
    if W * n_pkts < 1 << 22:
        for w in range(W):
            one(w)
    else:
        from concurrent.futures import ThreadPoolExecutor
        with ThreadPoolExecutor(max_workers=8) as ex:
            list(ex.map(one, range(W)))
    return out


def survive_microburst(seed, it, rnd, slot_of: np.ndarray, n_windows, window_frac, p_iid) -> np.ndarray:
    """Contiguous drop windows over the global wire sequence (slot space) plus i.i.d. loss.
    Window starts are drawn so the windows do not overlap."""
    W, n_pkts = slot_of.shape
    n_slots = W * n_pkts
    wlen = max(1, int(n_slots * window_frac))
    rng = np.random.Generator(np.random.PCG64(key(seed, STREAM_WINDOWS, it, rnd)))
    # place windows in distinct equal segments so they cannot overlap
    seg = n_slots // n_windows
    assert seg >= wlen
    starts = [j * seg + int(rng.integers(0, seg - wlen + 1)) for j in range(n_windows)]
    slot_survive = np.empty(n_slots, dtype=np.uint8)
    _cpu_lib().dblp_gen_bernoulli(slot_survive.ctypes.data, n_slots, key(seed, STREAM_LOSS, it, rnd, 0), q32(p_iid))
    for s in starts:
        slot_survive[s:s + wlen] = 0
    return slot_survive[slot_of.reshape(-1)].reshape(W, n_pkts)


# ----------------------------------------------------------------------------
# wire placement and arrival order
# ----------------------------------------------------------------------------
def placement(kind: str, W: int, n_pkts: int, seed: int, it: int = 0) -> np.ndarray:
    """slot_of[w, seq]: where packet (w, seq) sits in the wire/receive buffer.
    worker_major: worker w's packets contiguous, seq ascending.
    interleave:   each worker's packets keep seq order; the merge across workers is random.
    shuffle:      uniformly random slot for every packet."""
    n = W * n_pkts
    rng = np.random.Generator(np.random.PCG64(key(seed, STREAM_PLACE, it)))
    if kind == "worker_major":
        return np.arange(n, dtype=np.uint32).reshape(W, n_pkts)
    if kind == "shuffle":
        return rng.permutation(n).astype(np.uint32).reshape(W, n_pkts)
    if kind == "interleave":
        owner = np.repeat(np.arange(W, dtype=np.uint8), n_pkts)
        rng.shuffle(owner)                      # owner[s] = worker whose packet sits at slot s
        slots_sorted = np.argsort(owner, kind="stable").astype(np.uint32)  # worker-major list of slots, ascending
        return slots_sorted.reshape(W, n_pkts)
    raise ValueError(kind)


def arrival_order(kind: str, n_slots: int, seed: int, it: int = 0) -> np.ndarray | None:
    """order[k] = slot of the k-th arrival."""
    if kind == "identity":
        return None
    if kind == "shuffle":
        rng = np.random.Generator(np.random.PCG64(key(seed, STREAM_ORDER, it)))
        return rng.permutation(n_slots).astype(np.uint32)
    if kind == "reverse":
        return np.arange(n_slots - 1, -1, -1, dtype=np.uint32)
    raise ValueError(kind)


def chunk_seq_ranges(layout: "Layout", chunk_buckets: int):
    """[(seq0, seq1)] of consecutive groups of `chunk_buckets` buckets (one group if 0)."""
    if chunk_buckets <= 0:
        return [(0, layout.n_pkts)]
    fs = layout.first_seq
    return [(int(fs[b]), int(fs[min(b + chunk_buckets, layout.B)])) for b in range(0, layout.B, chunk_buckets)]


def placement_chunked(kind: str, layout: "Layout", chunk_buckets: int, seed: int, it: int = 0) -> np.ndarray:
    """Placement for chunk-streamed workloads: step c carries seq range [s0, s1) of every
    worker in its own contiguous slot range [W*s0, W*s1); `kind` applies inside each step."""
    W = layout.W
    slot_of = np.empty((W, layout.n_pkts), dtype=np.uint32)
    for c, (s0, s1) in enumerate(chunk_seq_ranges(layout, chunk_buckets)):
        slot_of[:, s0:s1] = placement(kind, W, s1 - s0, seed, it * 4096 + c) + np.uint32(W * s0)
    return slot_of


def slot_mask_words(survive: np.ndarray, slot_of: np.ndarray) -> np.ndarray:
    """Pack survival bits into 64-bit words indexed by slot (bit s%64 of word s//64)."""
    n_slots = slot_of.size
    by_slot = np.zeros((n_slots + 63) // 64 * 64, dtype=np.uint8)
    by_slot[slot_of.reshape(-1)] = survive.reshape(-1)
    return np.packbits(by_slot, bitorder="little").view(np.uint64).copy()


# ----------------------------------------------------------------------------
# named workloads
# ----------------------------------------------------------------------------
@dataclass
class Workload:
    name: str
    layout: Layout
    sigma: float
    loss: dict            # {"kind": "bernoulli"|"ge"|"microburst", ...}
    place: str            # placement kind
    order: str            # arrival-order kind
    policy: dict          # {"kind": "fixed"|"two_level"|"three_level"|"linear", ...}
    iterations: int = 1
    tail_ppm: int = 0
    tail_mul: float = 1.0
    chunk_buckets: int = 0   # >0: packets are applied in steps of this many buckets
    seed: int = MASTER_SEED
    scale_schedule: tuple = ()  # per-iteration multiplier on sigma (empty: all 1)
    drawn_rounds: int = 6       # retransmission rounds that draw loss; later rounds lose nothing

    def sigma_at(self, it: int) -> float:
        return self.sigma * (self.scale_schedule[it] if self.scale_schedule else 1.0)

    def survive(self, it: int, rnd: int, slot_of: np.ndarray | None = None) -> np.ndarray:
        L, k = self.layout, self.loss
        if k["kind"] == "none":
            return np.ones((L.W, L.n_pkts), dtype=np.uint8)
        if k["kind"] == "bernoulli":
            return survive_bernoulli(self.seed, it, rnd, L.W, L.n_pkts, k["p"])
        if k["kind"] == "ge":
            return survive_gilbert_elliott(self.seed, it, rnd, L.W, L.n_pkts, k["p_good"], k["p_bad"],
                                           k["p_g2b"], k["p_b2g"])
        if k["kind"] == "burst_iter":
            # the paper's microburst: a whole iteration (first transmission and every
            # retransmission round of it) suffers loss rate p_burst; other iterations p_bg
            p = k["p_burst"] if it in k["burst_iters"] else k["p_bg"]
            return survive_bernoulli(self.seed, it, rnd, L.W, L.n_pkts, p)
        if k["kind"] == "microburst":
            if rnd > 0:  # retransmissions see only the background loss
                return survive_bernoulli(self.seed, it, rnd, L.W, L.n_pkts, k["p_iid"])
            assert slot_of is not None
            return survive_microburst(self.seed, it, rnd, slot_of, k["n_windows"], k["window_frac"], k["p_iid"])
        raise ValueError(k["kind"])


def _decay_schedule(iters: int):
    """Smooth 0.97x decay with sharp drops at t=10,30 (x0.45) and a x0.7 step at t=20."""
    s, out = 1.0, []
    for t in range(iters):
        if t in (10, 30):
            s *= 0.45
        elif t == 20:
            s *= 0.7
        elif t > 0:
            s *= 0.97
        out.append(s)
    return tuple(out)


GE_BASE = dict(kind="ge", p_good=0.001, p_bad=0.30, p_g2b=1.0 / 1960.0, p_b2g=1.0 / 40.0)
GE_5X = dict(kind="ge", p_good=0.005, p_bad=0.30, p_g2b=5.0 / 1960.0, p_b2g=1.0 / 40.0)


def workload(name: str, seed: int = MASTER_SEED) -> Workload:
    if name == "cfg1":
        N, P, W = 1 << 20, 256, 4
        off, cnt = buckets_fixed(N, P, 64)
        return Workload(name, Layout(W, N, P, off, cnt), 1e-3, dict(kind="bernoulli", p=0.01),
                        "worker_major", "shuffle", dict(kind="fixed", ppm=50000), seed=seed)
    if name == "cfg2":
        N, P, W = 25_600_000, 366, 8
        off, cnt = buckets_from_sizes(sizes_loguniform(N, 161, 1000, 2_400_000, seed))
        return Workload(name, Layout(W, N, P, off, cnt), 1e-3, dict(kind="bernoulli", p=0.02),
                        "shuffle", "shuffle", dict(kind="fixed", ppm=50000), seed=seed)
    if name == "cfg3":
        sizes = sizes_gpt2(768, 12)
        off, cnt = buckets_from_sizes(sizes)
        return Workload(name, Layout(8, int(sizes.sum()), 366, off, cnt), 1e-3, dict(GE_BASE),
                        "shuffle", "shuffle",
                        dict(kind="three_level", ppm=(10000, 50000, 100000), eta=0.5),
                        iterations=50, scale_schedule=_decay_schedule(50), seed=seed)
    if name == "cfg4":
        sizes = sizes_gpt2(1024, 24)
        off, cnt = buckets_from_sizes(sizes)
        return Workload(name, Layout(16, int(sizes.sum()), 1024, off, cnt), 1e-3,
                        dict(kind="microburst", n_windows=3, window_frac=0.005, p_iid=0.005),
                        "interleave", "identity", dict(kind="fixed", ppm=80000), seed=seed)
    if name == "cfg5":
        N, P, W = 1_300_000_000, 366, 32
        off, cnt = buckets_fixed(N, P, 4096)
        return Workload(name, Layout(W, N, P, off, cnt), 1e-4, dict(GE_5X),
                        "shuffle", "shuffle",
                        dict(kind="linear", lo_ppm=20000, hi_ppm=150000, eta=0.5),
                        iterations=20, tail_ppm=10000, tail_mul=100.0, chunk_buckets=44,
                        scale_schedule=_decay_schedule(20), seed=seed)
    raise ValueError(name)


def paper_model_workload(name: str, burst_rate: float, burst_iters, iterations: int, seed: int = MASTER_SEED,
                         p_bg: float = 0.002) -> Workload:
    """The paper's own setting, as far as it is stated: 3 workers and one server, one accounting
    unit per worker and round (a single bucket), MTU-filling packets, parameter counts of Table 1.
    Whole-iteration microbursts at `burst_iters` with loss rate `burst_rate` (60-90 % in the paper);
    the background loss p_bg is this repository's choice (the paper's network is a black box)."""
    n_params = {"effnetb0": 5_288_548, "resnet50": 25_557_032, "alexnet": 61_100_840, "gpt2s": 124_439_808}[name]
    off, cnt = buckets_from_sizes([n_params])
    p_low = 24_000 if name == "resnet50" else 8_000
    return Workload(f"paper_{name}", Layout(3, n_params, 366, off, cnt), 1e-3,
                    dict(kind="burst_iter", p_bg=p_bg, p_burst=burst_rate, burst_iters=tuple(burst_iters)),
                    "interleave", "shuffle",
                    dict(kind="two_level", low_ppm=p_low, high_ppm=p_low + 400_000, eta=0.5),
                    iterations=iterations, seed=seed, drawn_rounds=1_000_000)


def scaled_down(wl: Workload, N: int, name: str | None = None) -> Workload:
    """Same recipe on a smaller gradient: keeps W, P, loss, placement and policy; bucket
    sizes are scaled to sum to N (fixed-size bucket tables keep their packets-per-bucket)."""
    L = wl.layout
    sizes = L.bucket_cnt.astype(np.float64)
    if np.all(L.bucket_cnt[:-1] == L.bucket_cnt[0]):
        off, cnt = buckets_fixed(N, L.P, int(L.n_b[0]))
    else:
        s = np.maximum(1, np.floor(sizes * (N / sizes.sum()))).astype(np.int64)
        s[-1] += N - s.sum()
        assert s.min() >= 1
        off, cnt = buckets_from_sizes(s)
    import dataclasses
    return dataclasses.replace(wl, name=name or f"{wl.name}_n{N}", layout=Layout(L.W, N, L.P, off, cnt))
