"""Test/bench harness: builds one scenario's inputs on the host and drives a receiver
(the CPU oracle or the GPU library, through small adapters) through one iteration:
begin_round -> apply_arrivals (per chunk step) -> loss_account -> simulated
retransmissions until every bucket meets the bound -> finalize -> phase_signal.

The harness holds no aggregation arithmetic; it only moves inputs and collects outputs.
"""
from __future__ import annotations

from dataclasses import dataclass, field

import numpy as np

import workloads as wl



@dataclass
class Batch:
    slot_base: int            # first slot of this arrival batch inside the packet buffer
    n_slots: int
    mask: np.ndarray | None   # uint64 words, bit s = local slot s survived (None: all)
    order: np.ndarray | None  # uint32 local slot per arrival (None: identity)


@dataclass
class Scenario:
    w: wl.Workload
    it: int
    rnd_id: int                       # round counter carried in headers
    slot_of: np.ndarray               # uint32 [W, n_pkts] global slot of each packet
    batches: list                     # first-transmission arrival batches
    survive0: np.ndarray              # uint8 [W, n_pkts]
    _survive_cache: dict = field(default_factory=dict)

    @property
    def L(self):
        return self.w.layout

    def grad(self, w: int, e0: int = 0, n: int | None = None) -> np.ndarray:
        n = self.L.N - e0 if n is None else n
        return wl.grad_values(self.w.seed, w, self.it, e0, n, self.w.sigma_at(self.it),
                              self.w.tail_ppm, self.w.tail_mul)

    def survive(self, rnd: int) -> np.ndarray:
        if rnd == 0:
            return self.survive0
        if rnd > self.w.drawn_rounds:
            return np.ones_like(self.survive0)
        if rnd not in self._survive_cache:
            self._survive_cache[rnd] = self.w.survive(self.it, rnd, self.slot_of)
        return self._survive_cache[rnd]

    def resend(self, retx_list: np.ndarray, rnd: int) -> np.ndarray:
        """Global slots of the listed packets that survive retransmission round `rnd`,
        in list order: the arrival order of the retransmission batch."""
        ws = (retx_list >> np.uint64(32)).astype(np.int64)
        seqs = (retx_list & np.uint64(0xFFFFFFFF)).astype(np.int64)
        ok = self.survive(rnd)[ws, seqs].astype(bool)
        return self.slot_of[ws[ok], seqs[ok]].astype(np.uint32)


def build_scenario(w: wl.Workload, it: int = 0, place: str | None = None, order: str | None = None) -> Scenario:
    L = w.layout
    place = place or w.place
    order = order or w.order
    slot_of = wl.placement_chunked(place, L, w.chunk_buckets, w.seed, it)
    survive0 = w.survive(it, 0, slot_of)
    batches = []
    for c, (s0, s1) in enumerate(wl.chunk_seq_ranges(L, w.chunk_buckets)):
        base, n = L.W * s0, L.W * (s1 - s0)
        local = (slot_of[:, s0:s1] - np.uint32(base)).astype(np.uint32)
        mask = wl.slot_mask_words(survive0[:, s0:s1], local)
        batches.append(Batch(base, n, mask, wl.arrival_order(order, n, w.seed, it * 4096 + c)))
    return Scenario(w, it, (it + 1) & 0xFFFF, slot_of, batches, survive0)


# ---------------------------------------------------------------------------------------
# oracle adapter
# ---------------------------------------------------------------------------------------
class OracleRx:
    """Drives oracle.Oracle on host packets."""

    def __init__(self, sc: Scenario, eta: float = 0.5, threads: int | None = None):
        """threads: None = the plain single-threaded walk; otherwise the element-range-parallel walk
        (same results, used to time the baseline on all cores; 0 = all that OpenMP offers)."""
        import oracle
        L = sc.L
        self.sc = sc
        self.threads, self.threads_used = threads, 1
        self.o = oracle.Oracle(L.W, L.N, L.P, L.bucket_off, L.bucket_cnt, eta)
        self.packets = None
        self.src = None

    def packetize_all(self, rnd_id: int | None = None):
        sc, L, o = self.sc, self.sc.L, self.o
        rnd_id = sc.rnd_id if rnd_id is None else rnd_id
        self.packets = np.zeros(L.W * L.n_pkts * L.stride, dtype=np.uint8)
        self.src = np.full(L.W * L.n_pkts, 0xFFFF, dtype=np.uint16)
        for w in range(L.W):
            o.packetize(w, rnd_id, sc.grad(w), 0, 0, L.n_pkts, self.packets, self.src, slot_map=sc.slot_of[w])

    def begin_round(self, rnd_id):
        self.o.begin_round(rnd_id)

    def apply(self, slot_base, n_slots, mask, order, n_arrivals=None):
        st = self.o.stride
        self.threads_used = self.o.apply_arrivals(self.packets[slot_base * st:], self.src[slot_base:], n_slots, mask,
                                                  order, n_arrivals, threads=self.threads)

    def loss_account(self, bound_ppm):
        return self.o.loss_account(bound_ppm)

    def finalize(self):
        self.out = self.o.finalize()
        return self.out

    def phase_signal(self):
        return self.o.phase_signal(self.out)

    def prev_norm(self):
        return self.o.get_prev_norm()

    def bitmap(self):
        return self.o.received()

    def counters(self):
        return self.o.counters()


def run_iteration(rx, sc: Scenario, bound_ppm: int, max_rounds: int = 256) -> dict:
    """One full iteration on receiver `rx`.  Returns everything observable."""
    L = sc.L
    rx.begin_round(sc.rnd_id)
    for b in sc.batches:
        rx.apply(b.slot_base, b.n_slots, b.mask, b.order)
    probes = []
    rnd = 0
    while True:
        missing, lst, count, met = rx.loss_account(bound_ppm)
        probes.append(dict(missing=np.array(missing, copy=True), list=np.array(lst, copy=True), count=count, met=met))
        if met:
            break
        rnd += 1
        assert rnd <= max_rounds, "retransmission did not converge"
        slots = sc.resend(lst, rnd)
        rx.apply(0, L.W * L.n_pkts, None, slots, slots.size)
    out = rx.finalize()
    prev = rx.prev_norm()
    norm, delta, crit = rx.phase_signal()
    return dict(probes=probes, rounds=rnd, bitmap=rx.bitmap(), out=out, norm=norm, rel_delta=delta,
                critical=crit, counters=rx.counters(), prev_norm=prev)


def definition_mean(sc: Scenario, received: np.ndarray) -> np.ndarray:
    """The one-line definition out[e] = (1/W) * sum_w received[w, pkt(e)] * g[w, e], in float64,
    written with numpy only (no oracle code): used to pin the oracle."""
    L = sc.L
    out = np.zeros(L.N, dtype=np.float64)
    pkt_of_elem = np.empty(L.N, dtype=np.int64)
    for b in range(L.B):
        off, cnt = int(L.bucket_off[b]), int(L.bucket_cnt[b])
        pkt_of_elem[off:off + cnt] = int(L.first_seq[b]) + np.arange(cnt) // L.P
    for w in range(L.W):
        out += received[w, pkt_of_elem].astype(np.float64) * sc.grad(w).astype(np.float64)
    return out / L.W


# ---------------------------------------------------------------------------------------
# GPU adapter (C-ABI library through its Python binding)
# ---------------------------------------------------------------------------------------
def _dev(a: np.ndarray, as_dtype):
    import torch
    return torch.from_numpy(np.ascontiguousarray(a).view(as_dtype)).cuda()


def receive_queue(src: np.ndarray, n_slots: int, mask, order, n_arrivals=None) -> np.ndarray:
    """The batch (per-slot worker table, survival mask, arrival order) as a receive queue: one
    descriptor slot | worker << 32 per arrival that survived, in arrival order.  Arrivals whose
    slot lies outside the buffer are kept (worker 0): the receiver must call them invalid."""
    if order is None:
        slots = np.arange(n_slots if n_arrivals is None else n_arrivals, dtype=np.uint64)
    else:
        slots = np.asarray(order, dtype=np.uint64)[:n_arrivals]
    inside = slots < n_slots
    keep = np.ones(slots.size, dtype=bool)
    if mask is not None:
        s_in = slots[inside]
        words = np.asarray(mask, dtype=np.uint64)
        keep[inside] = ((words[s_in >> np.uint64(6)] >> (s_in & np.uint64(63))) & np.uint64(1)).astype(bool)
    worker = np.zeros(slots.size, dtype=np.uint64)
    worker[inside] = np.asarray(src).astype(np.uint64)[slots[inside]]
    return (slots | (worker << np.uint64(32)))[keep]


class GpuRx:
    """Drives the HIP library on device-resident packets built by its own packetize."""

    def __init__(self, sc: Scenario, eta: float = 0.5, queue: bool = False, acc_copies: int = 1, acc_policy: int = 0,
                 acc_place: int = 0, result: str = "copy"):
        """queue=True hands every batch over as a receive queue (dblp_apply_arrivals_queue): the
        descriptors are built here, on the host, from the same (mask, order, per-slot worker).
        result: "copy" finalize writes a buffer of the caller's; "in_place" finalize(NULL), the result
        is read from the library's first accumulator copy; "caller" the accumulator copies are
        tensors owned here and finalize is given the first of them."""
        import torch
        import paper_2605_01989_amd as dblp
        L = sc.L
        self.sc, self.torch, self.queue, self.result = sc, torch, queue, result
        self.d_out = torch.empty(L.N, dtype=torch.float32, device="cuda")
        if result == "caller":
            self.d_second = torch.empty(L.N, dtype=torch.float32, device="cuda") if acc_copies == 2 else None
            self.agg = dblp.Aggregator(L.W, L.N, L.P, L.bucket_off, L.bucket_cnt, eta,
                                       accumulator_mode=1 if acc_copies == 2 else 0,
                                       d_accumulator=(self.d_out, self.d_second))
            self.agg.accumulator_policy(acc_policy)
        else:
            self.agg = dblp.Aggregator(L.W, L.N, L.P, L.bucket_off, L.bucket_cnt, eta)
            if acc_copies == 2:  # a second accumulator copy, and which copy batches write new spans to
                self.agg.accumulator_copies(2, place=acc_place)
                self.agg.accumulator_policy(acc_policy)
        assert (self.agg.n_pkts, self.agg.stride) == (L.n_pkts, L.stride)
        n_slots = L.W * L.n_pkts
        self.packets = torch.zeros(n_slots * L.stride, dtype=torch.uint8, device="cuda")
        self.src = torch.full((n_slots,), -1, dtype=torch.int16, device="cuda")
        self.d_missing = torch.empty(L.W * L.B, dtype=torch.int32, device="cuda")
        self.d_list = torch.empty(max(n_slots, 1), dtype=torch.int64, device="cuda")
        self.d_bitmap = torch.empty(L.W * self.agg.words_pw, dtype=torch.int64, device="cuda")

    def packetize_all(self, rnd_id: int | None = None):
        sc, L = self.sc, self.sc.L
        rnd_id = sc.rnd_id if rnd_id is None else rnd_id
        for w in range(L.W):
            d_grad = self.torch.from_numpy(sc.grad(w)).cuda()
            d_map = _dev(sc.slot_of[w], np.int32)
            self.agg.packetize(w, rnd_id, d_grad, 0, 0, L.n_pkts, self.packets, self.src, d_slot_map=d_map)

    def upload_packets(self, packets: np.ndarray, src: np.ndarray):
        """Use host-built wire bytes (e.g. with hand-corrupted headers) instead of packetize."""
        self.packets.copy_(self.torch.from_numpy(packets))
        self.src.copy_(self.torch.from_numpy(src.view(np.int16)))

    def begin_round(self, rnd_id):
        self.agg.begin_round(rnd_id)

    def _descriptors(self, slot_base, n_slots, mask, order, n_arrivals):
        src = self.src[slot_base: slot_base + n_slots].cpu().numpy().view(np.uint16)
        return receive_queue(src, n_slots, mask, order, n_arrivals)

    def apply(self, slot_base, n_slots, mask, order, n_arrivals=None):
        st = self.agg.stride
        if self.queue:
            q = self._descriptors(slot_base, n_slots, mask, order, n_arrivals)
            if q.size:
                self.agg.apply_arrivals_queue(self.packets[slot_base * st:], n_slots, _dev(q, np.int64), q.size)
            return
        d_mask = None if mask is None else _dev(mask, np.int64)
        d_order = None if order is None else _dev(np.asarray(order, dtype=np.uint32), np.int32)
        if order is not None and n_arrivals is None:
            n_arrivals = int(np.asarray(order).size)
        if d_order is not None and d_order.numel() == 0:
            d_order = None
            n_arrivals = 0
        self.agg.apply_arrivals(self.packets[slot_base * st:], self.src[slot_base:], n_slots, d_mask, d_order, n_arrivals)

    def loss_account(self, bound_ppm, capacity=None):
        L = self.sc.L
        count, met, trunc = self.agg.loss_account(bound_ppm, self.d_missing, self.d_list, capacity)
        n = min(count, self.d_list.numel() if capacity is None else capacity)
        missing = self.d_missing.cpu().numpy().view(np.uint32).reshape(L.W, L.B)
        return missing, self.d_list[:n].cpu().numpy().view(np.uint64), count, met

    def finalize(self):
        if self.result == "in_place":
            self.agg.finalize(None)
            return self.agg.accumulator_tensor(0).cpu().numpy()
        self.agg.finalize(self.d_out)        # "caller": d_out is the accumulator, so this is in place too
        return self.d_out.cpu().numpy()

    def phase_signal(self):
        return self.agg.phase_signal()

    def prev_norm(self):
        return self.agg.get_prev_norm()

    def bitmap(self):
        L = self.sc.L
        self.agg.get_bitmap(self.d_bitmap)
        words = self.d_bitmap.cpu().numpy().view(np.uint64).reshape(L.W, self.agg.words_pw)
        bits = np.unpackbits(words.view(np.uint8), axis=1, bitorder="little")
        assert not bits[:, L.n_pkts:].any(), "bitmap bits set beyond n_pkts"
        return bits[:, :L.n_pkts]

    def counters(self):
        return self.agg.get_counters()


def abs_scale(sc: Scenario, received: np.ndarray) -> np.ndarray:
    """(1/W) sum_w received[w, pkt(e)] |g[w, e]|: the natural scale of element e's sum, used as
    the denominator of the float parity metric (a relative error against the magnitude of the
    addends, which is what any summation order can guarantee)."""
    L = sc.L
    out = np.zeros(L.N, dtype=np.float64)
    pkt_of_elem = np.empty(L.N, dtype=np.int64)
    for b in range(L.B):
        off, cnt = int(L.bucket_off[b]), int(L.bucket_cnt[b])
        pkt_of_elem[off:off + cnt] = int(L.first_seq[b]) + np.arange(cnt) // L.P
    for w in range(L.W):
        out += received[w, pkt_of_elem].astype(np.float64) * np.abs(sc.grad(w).astype(np.float64))
    return out / L.W


FLOAT_TOL = 1e-5   # max relative error of the fp32 aggregate against the fp64 oracle


def record_stat(name: str, stats: dict) -> None:
    """Prints one parity record and, when DBLP_PARITY_STATS names a file, appends it there as a
    JSON line (the plain element-wise relative error and the count of elements above the
    tolerance are reported this way, next to the asserted metric)."""
    import json
    import os
    line = json.dumps(dict(case=name, **stats), default=lambda v: v.item() if hasattr(v, "item") else str(v))
    print(line, flush=True)
    path = os.environ.get("DBLP_PARITY_STATS")
    if path:
        with open(path, "a") as f:
            f.write(line + "\n")


def compare_results(got: dict, ref: dict, sc: Scenario) -> dict:
    """Integer outputs bit-exact; floats within FLOAT_TOL of the oracle relative to the addends'
    magnitude; never-received elements exactly zero; norm within 1e-6 of itself plus four fp32
    ulps of the addends' magnitude (in the 2-norm)."""
    assert np.array_equal(got["bitmap"], ref["bitmap"]), "bitmap differs"
    assert got["rounds"] == ref["rounds"]
    assert len(got["probes"]) == len(ref["probes"])
    for i, (a, b) in enumerate(zip(got["probes"], ref["probes"])):
        assert a["count"] == b["count"] and a["met"] == b["met"], f"probe {i}: count/met differ"
        assert np.array_equal(a["missing"], b["missing"]), f"probe {i}: missing counts differ"
        assert np.array_equal(a["list"], b["list"]), f"probe {i}: retransmit list differs"
    assert got["counters"] == ref["counters"], (got["counters"], ref["counters"])
    g, r = got["out"].astype(np.float64), ref["out"]
    scale = abs_scale(sc, ref["bitmap"])
    zero = scale == 0
    assert np.all(g[zero] == 0.0), "element that no worker delivered is not exactly zero"
    err = np.abs(g - r)
    rel = float((err[~zero] / scale[~zero]).max()) if (~zero).any() else 0.0
    assert rel <= FLOAT_TOL, f"float parity {rel:.3e} > {FLOAT_TOL}"
    nz = r != 0
    plain = err[nz] / np.abs(r[nz])
    assert got["critical"] == ref["critical"]
    norm_tol = 0.0
    if ref["norm"] > 0:
        # | ||gpu|| - ||oracle|| | <= ||gpu - oracle||_2: besides 1e-6 of the norm itself the fp32 result may
        # carry a few ulps of its ADDENDS' magnitude per element (the same cancellation that makes the
        # plain element-wise relative error meaningless: a one-element gradient whose 48 addends of
        # 1e-3 cancel to 3e-6 has a norm that is exact only to 4e-6 of itself)
        norm_tol = 1e-6 * ref["norm"] + 2.0 ** -22 * float(np.linalg.norm(scale))
        assert abs(got["norm"] - ref["norm"]) <= norm_tol, (got["norm"], ref["norm"], norm_tol)
    # Eq. 1 on each side's own norms: the reported change must be |prev - cur| / prev of the norms
    # that side holds; the two sides' values then differ by no more than their norms explain
    for side in (got, ref):
        p = side.get("prev_norm")
        if p:
            want = abs(p - side["norm"]) / p
            assert abs(side["rel_delta"] - want) <= 1e-12 * max(1.0, want), (side["rel_delta"], want)
        else:
            assert np.isinf(side["rel_delta"]) and side["critical"]
    if np.isfinite(ref["rel_delta"]):
        slack = norm_tol / ref["norm"] if ref["norm"] > 0 else 0.0
        if got.get("prev_norm") and ref.get("prev_norm"):
            slack += abs(got["prev_norm"] - ref["prev_norm"]) / ref["prev_norm"]
        assert abs(got["rel_delta"] - ref["rel_delta"]) <= 1e-5 + 2.0 * (1.0 + ref["rel_delta"]) * slack
    else:
        assert got["rel_delta"] == ref["rel_delta"]
    return dict(rel_to_addends=rel, rel_to_max=float(err.max() / max(np.abs(r).max(), 1e-300)),
                plain_rel_max=float(plain.max()) if nz.any() else 0.0,
                plain_rel_above_tol=int((plain > FLOAT_TOL).sum()), n=int(r.size))
