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

MAX_DRAWN_ROUNDS = 6   # retransmission rounds with a drawn loss pattern; later rounds lose nothing


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
        if rnd > MAX_DRAWN_ROUNDS:
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

    def __init__(self, sc: Scenario, eta: float = 0.5):
        import oracle
        L = sc.L
        self.sc = sc
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
        self.o.apply_arrivals(self.packets[slot_base * st:], self.src[slot_base:], n_slots, mask, order, n_arrivals)

    def loss_account(self, bound_ppm):
        return self.o.loss_account(bound_ppm)

    def finalize(self):
        self.out = self.o.finalize()
        return self.out

    def phase_signal(self):
        return self.o.phase_signal(self.out)

    def bitmap(self):
        return self.o.received()

    def counters(self):
        return self.o.counters()


def run_iteration(rx, sc: Scenario, bound_ppm: int, max_rounds: int = 64) -> dict:
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
    norm, delta, crit = rx.phase_signal()
    return dict(probes=probes, rounds=rnd, bitmap=rx.bitmap(), out=out, norm=norm, rel_delta=delta,
                critical=crit, counters=rx.counters())


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
