#!/usr/bin/env python3
"""Benchmark of the DBLP receiver hot path on one MI355X.

A step is one full iteration of the receiver over one round of synthetic input that is
already resident in HBM: begin_round -> apply_arrivals (one call per chunk step) ->
loss_account -> simulated retransmissions until every (worker, bucket) meets the bound ->
finalize -> phase_signal -> next bound.  Packetisation, gradient generation and loss-mask
generation happen before the timed region.

Prints ONE JSON line (see --help for the knobs).  `value` is aggregated gradient GB/s:
accepted payload bytes / wall time of the timed steps.
"""
from __future__ import annotations

import argparse
import hashlib
import json
import os
import sys
import time

ROOT = os.path.dirname(os.path.abspath(__file__))
for p in (ROOT, os.path.join(ROOT, "tests")):
    if p not in sys.path:
        sys.path.insert(0, p)

import numpy as np  # noqa: E402

HBM_PEAK_GBPS = 8000.0   # MI355X HBM3E, published peak
BENCH_DRAWN_ROUNDS = 3   # retransmission rounds with a drawn loss pattern; later rounds lose nothing

# HBM traffic of the dominant kernel measured with rocprofv3 --pmc (FETCH_SIZE x 2.00 + WRITE_SIZE,
# the factors calibrated on a 1 GiB copy), keyed by the SHA-256 of the kernel source it was measured
# on and by workload; anything else reports null.
# value = measured bytes / algorithmic bytes of a first-transmission launch.
PMC_TRAFFIC_RATIO: dict[tuple[str, str], float] = {
    ("3d4a1fc4cec74112deff2e5e7730b9e8e47595d4a41a9e5ff7a7fd105506a6c6", "cfg5"): 1.066,   # profiles/receiver_path_cfg5.md
    ("3d4a1fc4cec74112deff2e5e7730b9e8e47595d4a41a9e5ff7a7fd105506a6c6", "cfg4"): 1.030,   # profiles/receiver_path_cfg4.md
}


def _kernel_source_hash() -> str:
    src = os.path.join(ROOT, "paper_2605_01989_amd", "csrc", "dblp_agg.hip")
    return hashlib.sha256(open(src, "rb").read()).hexdigest()


def log(*a):
    print(*a, file=sys.stderr, flush=True)


class DeviceJob:
    """One workload with every input resident in HBM, driven through the C-ABI binding."""

    def __init__(self, w, n_masks: int, place: str | None = None, order: str | None = None, queue: bool = True,
                 accumulator: str = "one", both_forms_its=(),
                 drawn_rounds: int = BENCH_DRAWN_ROUNDS, per_iteration_retx: bool = False):
        """accumulator: "one" a single accumulator copy; "pair" a plain second copy; "search" a second
        copy searched for in another third of HBM (bounded: three fifths of the free memory, 8 s).
        The result is always left in place (finalize with no output buffer): d_out is a view of the
        library's first accumulator copy.
        both_forms_its: iterations whose first transmissions are prepared in both hand-over forms.
        drawn_rounds: retransmission rounds whose loss is drawn once (keyed to iteration 0) and kept
        on the device.  per_iteration_retx: draw every retransmission round's loss for the iteration
        at hand instead (small workloads whose loss process depends on the iteration)."""
        import torch
        import paper_2605_01989_amd as dblp
        import workloads as wl
        from paper_2605_01989_amd import binding
        self.torch, self.wl, self.w = torch, wl, w
        L = self.L = w.layout
        self.place, self.order = place or w.place, order or w.order
        self.queue = queue   # first transmissions handed over as receive queues (else mask + order + worker table)
        self.both_forms_its = set(both_forms_its)
        self.picks = None    # a list here collects the accumulator copy each receive-queue batch wrote new spans to
        self.rnd_id = 1
        mode = dict(one=binding.ACCMODE_SINGLE, trial=binding.ACCMODE_SINGLE, pair=binding.ACCMODE_PAIR,
                    search=binding.ACCMODE_SEARCH)[accumulator]
        self.agg = dblp.Aggregator(L.W, L.N, L.P, L.bucket_off, L.bucket_cnt, w.policy.get("eta", 0.5),
                                   accumulator_mode=mode, search_free_fraction=0.6, search_seconds=8.0)
        self.n_slots = L.W * L.n_pkts
        dev = "cuda"
        t0 = time.time()
        self.packets = torch.empty(self.n_slots * L.stride, dtype=torch.uint8, device=dev)
        self.src = torch.empty(self.n_slots, dtype=torch.int16, device=dev)
        # W a power of two: the result is left in place (d_out is a view of the first accumulator copy);
        # otherwise the library has to divide, which it does into a buffer of the caller's
        self.in_place = (L.W & (L.W - 1)) == 0
        self.d_out = self.agg.accumulator_tensor(0) if self.in_place else torch.empty(L.N, dtype=torch.float32, device=dev)
        self.d_missing = torch.empty(L.W * L.B, dtype=torch.int32, device=dev)
        self.list_cap = max(self.n_slots // 8, 1 << 16)
        self.d_list = torch.empty(self.list_cap, dtype=torch.int64, device=dev)
        self.d_resend = torch.empty(self.list_cap, dtype=torch.int32, device=dev)    # slots of the packets sent again
        self.stream = torch.cuda.current_stream().cuda_stream
        # placement and arrival orders (host generated, seeded)
        self.slot_of = wl.placement_chunked(self.place, L, w.chunk_buckets, w.seed, 0)
        self.d_slot_of = torch.from_numpy(self.slot_of.reshape(-1).view(np.int32)).to(dev)
        self.chunks = []
        for c, (s0, s1) in enumerate(wl.chunk_seq_ranges(L, w.chunk_buckets)):
            n = L.W * (s1 - s0)
            o = wl.arrival_order(self.order, n, w.seed, c)
            d_o = None if o is None else torch.from_numpy(o.view(np.int32)).to(dev)
            self.chunks.append(dict(s0=s0, s1=s1, base=L.W * s0, n=n, d_order=d_o))
        log(f"[bench] placement/order ready {time.time() - t0:.1f}s")
        self._generate_packets()
        log(f"[bench] packets resident {time.time() - t0:.1f}s ({self.packets.numel() / 1e9:.1f} GB)")
        # first-transmission masks per step, retransmission survival per drawn round
        self.masks = [self._mask_for(it) for it in range(n_masks)]
        self.d_survive = {}
        self.per_iteration_retx = per_iteration_retx
        self.d_survive_words = {}    # the same per slot, as mask words over the whole buffer
        for r in range(1, 0 if per_iteration_retx else drawn_rounds + 1):
            s = w.survive(0, r, self.slot_of)
            self.d_survive[r] = torch.from_numpy(s.reshape(-1)).to(dev)
            by_slot = torch.zeros(self.n_slots, dtype=torch.uint8, device=dev)
            by_slot[self.d_slot_of.long()] = self.d_survive[r]
            self.d_survive_words[r] = self._pack_bits(by_slot)
            del by_slot
        torch.cuda.synchronize()
        log(f"[bench] masks ready {time.time() - t0:.1f}s")

    # -- input preparation (outside the timed region) ------------------------------------
    def _generate_packets(self):
        torch, wl, w, L = self.torch, self.wl, self.w, self.L
        stream = torch.cuda.current_stream().cuda_stream
        max_elems = 0
        for ch in self.chunks:
            b0 = int(np.searchsorted(L.first_seq, ch["s0"], side="right") - 1)
            b1 = int(np.searchsorted(L.first_seq, ch["s1"] - 1, side="right") - 1)
            ch["e0"] = int(L.bucket_off[b0])
            ch["e1"] = int(L.bucket_off[b1] + L.bucket_cnt[b1])
            max_elems = max(max_elems, ch["e1"] - ch["e0"])
        grad = torch.empty(max_elems, dtype=torch.float32, device="cuda")
        for ch in self.chunks:
            ne = ch["e1"] - ch["e0"]
            for wk in range(L.W):
                wl.grad_fill_device(grad.data_ptr(), w.seed, wk, 0, ch["e0"], ne, w.sigma_at(0),
                                    w.tail_ppm, w.tail_mul, stream)
                d_map = self.d_slot_of[wk * L.n_pkts + ch["s0"]: wk * L.n_pkts + ch["s1"]]
                self.agg.packetize(wk, self.rnd_id, grad[:ne], ch["e0"], ch["s0"], ch["s1"] - ch["s0"],
                                   self.packets, self.src, d_slot_map=d_map, n_slots=self.n_slots)
        del grad

    def _pack_bits(self, bits):
        torch = self.torch
        n = bits.numel()
        pad = (-n) % 64
        if pad:
            bits = torch.cat([bits, torch.zeros(pad, dtype=torch.uint8, device=bits.device)])
        weights = torch.tensor([1, 2, 4, 8, 16, 32, 64, 128], dtype=torch.uint8, device=bits.device)
        return (bits.view(-1, 8) * weights).sum(dim=1, dtype=torch.uint8).view(torch.int64)

    def _mask_for(self, it: int):
        """Per chunk step: 64-bit words, bit s = local slot s survived the first transmission."""
        torch = self.torch
        surv = self.w.survive(it, 0, self.slot_of)
        d_s = torch.from_numpy(surv.reshape(-1)).cuda()
        by_slot = torch.zeros(self.n_slots, dtype=torch.uint8, device="cuda")
        by_slot[self.d_slot_of.long()] = d_s
        m = dict(lost=int(surv.size - int(surv.sum())))
        both = it in self.both_forms_its
        if self.queue or both:
            m["queues"] = [self._queue_for(ch, by_slot[ch["base"]: ch["base"] + ch["n"]]) for ch in self.chunks]
        if not self.queue or both:
            m["words"] = [self._pack_bits(by_slot[ch["base"]: ch["base"] + ch["n"]]) for ch in self.chunks]
        return m

    def _queue_for(self, ch, alive):
        """Receive queue of one chunk step: slot | worker << 32 for every packet that survived,
        in arrival order (what the mask, the order and the per-slot worker table say together)."""
        torch = self.torch
        o = ch["d_order"]
        slots = torch.arange(ch["n"], device="cuda") if o is None else o.long()
        slots = slots[alive[slots].bool()]
        worker = self.src[ch["base"]: ch["base"] + ch["n"]][slots].long() & 0xFFFF
        return slots | (worker << 32)

    def sender_timing(self, reps: int = 5) -> dict:
        """Sender side (Alg. "DBLP Send"), timed on its own and never part of `value`: the range
        packetiser on the first chunk step of every worker (the resident packets are rewritten with
        the bytes they already hold), and the list packetiser on the retransmit list that a probe
        with bound 0 gives after that chunk step alone.  Algorithmic bytes per packet: 4*len read +
        stride written."""
        torch, wl, w, L, agg = self.torch, self.wl, self.w, self.L, self.agg
        stream = torch.cuda.current_stream().cuda_stream
        ch = self.chunks[0]
        ne, npk = ch["e1"] - ch["e0"], ch["s1"] - ch["s0"]
        grads = []
        for wk in range(L.W):
            g = torch.empty(ne, dtype=torch.float32, device="cuda")
            wl.grad_fill_device(g.data_ptr(), w.seed, wk, 0, ch["e0"], ne, w.sigma_at(0), w.tail_ppm, w.tail_mul, stream)
            grads.append(g)
        maps = [self.d_slot_of[wk * L.n_pkts + ch["s0"]: wk * L.n_pkts + ch["s1"]] for wk in range(L.W)]
        ev = [torch.cuda.Event(enable_timing=True) for _ in range(2)]
        out = {}

        def timed(fn, n_bytes, n_calls):
            fn()
            torch.cuda.synchronize()
            ev[0].record()
            for _ in range(reps):
                fn()
            ev[1].record()
            torch.cuda.synchronize()
            ms = ev[0].elapsed_time(ev[1]) / reps
            return dict(GBps=round(n_bytes / ms / 1e6, 1), hbm_frac=round(n_bytes / ms / 1e6 / HBM_PEAK_GBPS, 4),
                        ms=round(ms, 4), calls=n_calls, algorithmic_bytes=int(n_bytes))

        def all_workers():
            for wk in range(L.W):
                agg.packetize(wk, self.rnd_id, grads[wk], ch["e0"], ch["s0"], npk, self.packets, self.src,
                              d_slot_map=maps[wk], n_slots=self.n_slots)
        out["packetize"] = timed(all_workers, L.W * (4 * ne + npk * L.stride), L.W)
        if ch["e0"] == 0:
            # a long retransmit list over this chunk step's sequence range: every fourth packet of every worker
            seqs = torch.arange(ch["s0"], ch["s1"], 4, device="cuda", dtype=torch.int64)
            lst = (torch.arange(L.W, device="cuda", dtype=torch.int64)[:, None] << 32 | seqs[None, :]).reshape(-1).contiguous()
            n = int(lst.numel())
            stage = torch.empty(n * L.stride, dtype=torch.uint8, device="cuda")
            stage_src = torch.empty(n, dtype=torch.int16, device="cuda")
            fill = L.N / (L.n_pkts * L.P)
            out["packetize_list"] = timed(lambda: agg.packetize_list(self.rnd_id, grads, lst, n, stage, stage_src),
                                          n * (4 * L.P * fill + L.stride), 1)
            out["packetize_list"]["entries"] = n
        return out

    def use_single_accumulator(self):
        """Switch the context to one accumulator copy (d_out is a view of it: refreshed here)."""
        if self.in_place:
            self.d_out = None                 # the view of the copy that is about to be released
        self.agg.accumulator_copies(1)
        if self.in_place:
            self.d_out = self.agg.accumulator_tensor(0)

    # -- the timed path --------------------------------------------------------------------
    def step(self, it: int, bound_ppm: int, scale_ratio: float = 1.0, record: list | None = None) -> dict:
        """One iteration.  scale_ratio = s_{t-1}/s_t of the workload's gradient-scale schedule:
        the resident gradient is not rescaled between steps, so the previous norm is rescaled
        instead, which gives Eq. 1 the same relative change.  With `record` (a list) every
        probe's per-bucket counts and retransmit list are copied to the host and appended."""
        torch, agg, L = self.torch, self.agg, self.L
        st = L.stride
        m = self.masks[it % len(self.masks)]
        agg.begin_round(self.rnd_id)
        if self.queue:
            for ch, q in zip(self.chunks, m["queues"]):
                agg.apply_arrivals_queue(self.packets[ch["base"] * st:], ch["n"], q)
                if self.picks is not None:
                    self.picks.append(agg.accumulator_info()["last_pick"])
        else:
            for ch, words in zip(self.chunks, m["words"]):
                agg.apply_arrivals(self.packets[ch["base"] * st:], self.src[ch["base"]:], ch["n"], words,
                                   ch["d_order"], ch["n"])
        rounds, resent = 0, 0
        while True:
            count, met, trunc = agg.loss_account(bound_ppm, self.d_missing, self.d_list)
            if trunc:
                raise RuntimeError(f"retransmit list ({count}) exceeds its buffer ({self.list_cap})")
            if record is not None:
                record.append(dict(count=count, met=met,
                                   missing=self.d_missing.cpu().numpy().view(np.uint32).reshape(L.W, L.B).copy(),
                                   list=self.d_list[:count].cpu().numpy().view(np.uint64).copy()))
            if met:
                break
            rounds += 1
            # the simulated sender + network: resend the listed packets, redraw their loss
            self.wl.resend_slots_device(self.d_list.data_ptr(), count, self.d_slot_of.data_ptr(), L.n_pkts,
                                        self.d_resend.data_ptr(), self.stream)
            if self.per_iteration_retx and rounds <= self.w.drawn_rounds:
                d_s = torch.from_numpy(self.w.survive(it, rounds, self.slot_of).reshape(-1)).cuda()
                lst = self.d_list[:count]
                idx = (lst >> 32) * L.n_pkts + (lst & 0xFFFFFFFF)
                slots = self.d_resend[:count][d_s[idx].bool()]
                resent += int(slots.numel())
                agg.apply_arrivals(self.packets, self.src, self.n_slots, None, slots, slots.numel())
            else:
                # every listed packet is sent again; the ones this round's loss draw takes are masked
                # out (lost on the wire: never looked at).  No host round trip besides the probe's.
                words = self.d_survive_words.get(rounds)
                agg.apply_arrivals(self.packets, self.src, self.n_slots, words, self.d_resend, count)
                if words is not None:
                    resent = None          # survivors not counted here: the caller derives them from the accepted counter
                elif resent is not None:
                    resent += count        # a round without drawn loss: everything arrives
        agg.finalize(None if self.in_place else self.d_out)     # in place: the result is the first accumulator copy
        prev = agg.get_prev_norm()
        if prev is not None:
            agg.set_prev_norm(prev * scale_ratio)
        norm, delta, crit = agg.phase_signal()
        return dict(rounds=rounds, resent=resent, norm=norm, rel_delta=delta, critical=crit, lost_first=m["lost"])


def place_accumulator_by_trial(job, w, n_candidates: int = 8, hold_fraction: float = 0.8) -> dict:
    """Set-up, before any timed step: where the accumulator lies relative to the resident packets
    decides several percent of the step, and only a measurement can tell (the physical layout of an
    allocation cannot be asked for).  So the caller does what a long-running receiver would do at
    start-up: it offers the library caller-owned accumulators at several places (buffers spread over
    the free memory, at most hold_fraction of it held at once), runs one untimed and one timed
    step with each, the library's own allocation included, and keeps the fastest.  The
    library is not involved beyond accepting the caller's buffer."""
    import torch
    import paper_2605_01989_amd as dblp
    from paper_2605_01989_amd import binding
    L = job.L
    n_bytes = 4 * L.N
    ctx_bytes = int(1.25 * 8 * L.W * L.n_pkts) + (64 << 20)       # a context's arrival index and small tables
    budget = int(torch.cuda.mem_get_info()[0] * hold_fraction)
    k_max = min(n_candidates, budget // (n_bytes + ctx_bytes))
    gap = max(0, (budget - k_max * (n_bytes + ctx_bytes)) // max(k_max, 1)) & ~((2 << 20) - 1)

    def timed_step():
        job.next_bound = first_bound(w)
        run_leg(job, w, [0])
        return run_leg(job, w, [0])["event_ms"]

    tried = [dict(where="library", ms=round(timed_step(), 3), agg=job.agg, acc=None)]
    fillers = []
    for k in range(k_max):
        try:
            acc = torch.empty(L.N, dtype=torch.float32, device="cuda")
            agg = dblp.Aggregator(L.W, L.N, L.P, L.bucket_off, L.bucket_cnt, w.policy.get("eta", 0.5),
                                  accumulator_mode=binding.ACCMODE_SINGLE, d_accumulator=(acc, None))
        except (RuntimeError, dblp.DblpError) as e:      # out of memory: make do with the places tried so far
            log(f"[bench] accumulator trial stops after {k} places: {e}")
            break
        job.agg = agg
        if job.in_place:
            job.d_out = acc
        tried.append(dict(where=f"{(acc.data_ptr() - job.packets.data_ptr()) / 2**30:+.1f} GiB from the packets",
                          ms=round(timed_step(), 3), agg=agg, acc=acc))
        if gap:
            try:
                fillers.append(torch.empty(gap, dtype=torch.uint8, device="cuda"))
            except RuntimeError:
                break
    best = min(tried, key=lambda t: t["ms"])
    job.agg = best["agg"]
    if job.in_place:
        job.d_out = best["acc"] if best["acc"] is not None else job.agg.accumulator_tensor(0)
    report = dict(candidates=[dict(where=t["where"], ms=t["ms"]) for t in tried], adopted=best["where"])
    job.plain_agg = tried[0]["agg"] if tried[0] is not best else None    # kept for the single-plain-copy leg of other_forms
    for t in tried[1:]:
        if t is not best:
            t["agg"] = t["acc"] = None
    del tried, fillers
    torch.cuda.empty_cache()
    return report


def default_accumulator(w) -> str:
    """Placing the accumulator by trial pays when one round carries at least 2 GiB of packets."""
    L = w.layout
    return "trial" if L.W * L.n_pkts * L.stride >= 2 << 30 else "one"


def next_bound(w, rel_delta: float, critical: bool) -> int:
    import paper_2605_01989_amd as dblp
    p = w.policy
    if p["kind"] == "fixed":
        return p["ppm"]
    if p["kind"] == "two_level":
        return dblp.policy_two_level(critical, p["low_ppm"], p["high_ppm"])
    if p["kind"] == "three_level":
        return dblp.policy_three_level(rel_delta, p["eta"], *p["ppm"])
    if p["kind"] == "linear":
        return dblp.policy_linear(rel_delta, p["eta"], p["lo_ppm"], p["hi_ppm"])
    raise ValueError(p["kind"])


def first_bound(w) -> int:
    p = w.policy
    return {"fixed": lambda: p["ppm"], "two_level": lambda: p["low_ppm"],
            "three_level": lambda: p["ppm"][0], "linear": lambda: p["lo_ppm"]}[p["kind"]]()


def host_description() -> dict:
    model = "unknown"
    try:
        for line in open("/proc/cpuinfo"):
            if line.lower().startswith("model name"):
                model = line.split(":", 1)[1].strip()
                break
    except OSError:
        pass
    try:
        usable = len(os.sched_getaffinity(0))
    except AttributeError:
        usable = os.cpu_count()
    return dict(cpu_model=model, nproc=os.cpu_count(), usable_cores=usable,
                omp_num_threads=os.environ.get("OMP_NUM_THREADS"))


def cpu_baseline(w, target_elems: int) -> dict:
    """The oracle, as it stands, timed on this host on a bounded sample of the same workload:
    same W, P, bucket shape, loss process, placement and order, smaller gradient.  Timed twice:
    the plain single-threaded walk (`value`) and the same arithmetic spread over all cores by
    element range (`all_cores`)."""
    import workloads as wl
    from harness import OracleRx, build_scenario, run_iteration
    ws = w if w.layout.N <= target_elems else wl.scaled_down(w, target_elems)
    sc = build_scenario(ws, 0)
    L = ws.layout
    fill = L.N / (L.n_pkts * L.P)
    rx = OracleRx(sc)
    rx.packetize_all()
    t0 = time.perf_counter()
    res = run_iteration(rx, sc, first_bound(ws))
    dt = time.perf_counter() - t0
    payload = res["counters"]["accepted"] * 4 * L.P * fill
    rx.threads = 0                                  # all cores OpenMP offers; same inputs, same receiver object
    t0 = time.perf_counter()
    res_mt = run_iteration(rx, sc, first_bound(ws))
    dt_mt = time.perf_counter() - t0
    assert res_mt["counters"] == res["counters"] and np.array_equal(res_mt["out"], res["out"])
    return dict(value=payload / dt / 1e9, unit="GB/s", cores=1, kind="oracle",
                sample=f"{ws.name}: W={L.W} N={L.N} P={L.P} packets={L.W * L.n_pkts} one iteration "
                       f"incl. {res['rounds']} retransmission round(s), {dt:.2f} s single-threaded, "
                       f"{dt_mt:.2f} s on {rx.threads_used} threads",
                packets_per_s=res["counters"]["accepted"] / dt,
                all_cores=dict(value=payload / dt_mt / 1e9, unit="GB/s", cores=rx.threads_used,
                               packets_per_s=res["counters"]["accepted"] / dt_mt,
                               note="arrival walk split by element range over the threads; finalize and the "
                                    "norm stay single-threaded"),
                host=host_description())


def run_leg(job, w, its, bounds=None, profile=False) -> dict:
    """Times the steps `its` (iteration numbers).  bounds: None = the workload's policy decides, starting
    from `job.next_bound`; a dict iteration -> bound replays a recorded run (the same work again).
    profile: False, True (every kernel group bracketed by events) or a bit mask of kernel groups."""
    import torch
    from paper_2605_01989_amd import binding
    agg = job.agg
    sched = w.scale_schedule

    def ratio(t):
        """s_{t-1}/s_t of the gradient-scale schedule (1 at its start and when there is none)."""
        if not sched or t % len(sched) == 0:
            return 1.0
        return sched[t % len(sched) - 1] / sched[t % len(sched)]

    if profile:
        agg.profile_enable(profile)
        for k in range(binding.K_COUNT):
            agg.profile_read(k)
    torch.cuda.synchronize()
    accepted_total, resent_total, rounds_total = 0, 0, 0
    ev0, ev1 = torch.cuda.Event(enable_timing=True), torch.cuda.Event(enable_timing=True)
    t_wall0 = time.perf_counter()
    ev0.record()
    per_step = []
    for t in its:
        bound = job.next_bound if bounds is None else bounds[t]
        r = job.step(t, bound, ratio(t))
        c = agg.get_counters()
        accepted_total += c["accepted"]
        # packets that arrived in retransmission rounds = accepted - first-transmission survivors
        resent = r["resent"] if r["resent"] is not None else c["accepted"] - (job.n_slots - r["lost_first"])
        resent_total += resent
        rounds_total += r["rounds"]
        per_step.append(dict(it=t, bound_ppm=bound, rounds=r["rounds"], resent=resent, accepted=c["accepted"]))
        job.next_bound = next_bound(w, r["rel_delta"], r["critical"])
    ev1.record()
    torch.cuda.synchronize()
    wall = time.perf_counter() - t_wall0
    out = dict(wall=wall, steps=len(its), accepted=accepted_total, resent=resent_total, rounds=rounds_total,
               per_step=per_step, event_ms=ev0.elapsed_time(ev1))
    if profile:
        out["prof"] = {name: agg.profile_read(k) for name, k in
                       (("index", binding.K_INDEX), ("gather", binding.K_GATHER), ("gather_direct", binding.K_GATHER_DIRECT),
                        ("probe", binding.K_PROBE), ("finalize", binding.K_FINALIZE))}
        agg.profile_enable(False)
    return out


def main():
    ap = argparse.ArgumentParser(description=__doc__)
    ap.add_argument("--gpus", type=int, default=1)
    ap.add_argument("--steps", type=int, default=10)
    ap.add_argument("--warmup", type=int, default=3)
    ap.add_argument("--workload", default="cfg5", help="cfg1..cfg5 (default: the largest, cfg5)")
    ap.add_argument("--place", default=None, help="override wire placement: worker_major|interleave|shuffle")
    ap.add_argument("--order", default=None, help="override arrival order: identity|shuffle|reverse")
    ap.add_argument("--arrivals", default="queue", choices=["queue", "tables"],
                    help="how first transmissions are handed over: one receive queue of descriptors per "
                         "chunk step (default), or mask + order + per-slot worker table")
    ap.add_argument("--accumulator", default=None, choices=["search", "pair", "one", "trial"],
                    help="search: a second accumulator copy is searched for in another third of HBM (bounded; "
                         "one copy when none is found); pair: a plain second copy; one: a single copy; trial: a "
                         "single caller-owned copy at the best of several places, found by timing one step with each "
                         "before the warm-up.  "
                         "Default: trial when a round carries at least 2 GiB of packets, else one")
    ap.add_argument("--extra-steps", type=int, default=5,
                    help="steps of the timed run that are replayed (same masks, same bounds) with the other "
                         "hand-over form and with a single accumulator copy, reported under other_forms; 0 = none")
    ap.add_argument("--no-cpu-baseline", action="store_true")
    ap.add_argument("--calibrate-copy", action="store_true",
                    help="also run one plain 1 GiB device-to-device copy (a kernel of known traffic, "
                         "to scale rocprofv3's FETCH_SIZE / WRITE_SIZE readings)")
    ap.add_argument("--cpu-sample-bytes", type=float, default=24e9,
                    help="packet bytes of the sample the CPU oracle is timed on (the workload scaled down "
                         "to that many bytes of first transmissions; about 10 s of single-threaded work)")
    args = ap.parse_args()
    if args.gpus != 1:
        sys.exit("bench.py: this library runs on one GPU only (all workers are simulated in that GPU's "
                 "memory); --gpus must be 1")

    import torch
    import workloads as wl
    assert torch.cuda.is_available(), "bench.py needs a GPU"
    torch.cuda.set_device(0)
    w = wl.workload(args.workload)
    L = w.layout
    if args.accumulator is None:
        args.accumulator = default_accumulator(w)
    total = args.warmup + args.steps
    n_extra = min(args.extra_steps, args.steps)
    extra_its = list(range(args.warmup, args.warmup + n_extra))
    form = {"queue": True, "tables": False}
    job = DeviceJob(w, n_masks=total, place=args.place, order=args.order, queue=form[args.arrivals],
                    accumulator=args.accumulator, both_forms_its=extra_its)
    trial = None
    if args.accumulator == "trial":
        trial = place_accumulator_by_trial(job, w)
        for t in trial["candidates"]:
            log(f"[bench] accumulator trial: {t['where']}: {t['ms']} ms")
    agg = job.agg

    if args.calibrate_copy:
        a = torch.ones(1 << 28, dtype=torch.float32, device="cuda")
        b = torch.empty_like(a)
        b.copy_(a)          # reads 1 GiB, writes 1 GiB
        torch.cuda.synchronize()
        del a, b
    sender = job.sender_timing()
    job.next_bound = first_bound(w)
    job.picks = []
    warm = run_leg(job, w, list(range(args.warmup)))
    picks, job.picks = job.picks[:len(job.chunks)], None
    for st in warm["per_step"]:
        log(f"[bench] warmup {st['it']}: bound={st['bound_ppm']} rounds={st['rounds']}")
    from paper_2605_01989_amd import binding
    # the timed region brackets only the launches of the dominant kernel, the staged gather, with events
    # (two event records per dense batch; the direct kernel's launches on sparse retransmission batches
    # are a group of their own); the per-group breakdown comes from a replay of its first steps with
    # every group bracketed
    main_leg = run_leg(job, w, list(range(args.warmup, total)), profile=1 << binding.K_GATHER)
    wall, prof = main_leg["wall"], main_leg["prof"]
    accepted_total = main_leg["accepted"]
    ms_per_step = wall * 1e3 / args.steps

    fill = L.N / (L.n_pkts * L.P)
    value = accepted_total * 4 * L.P * fill / wall / 1e9
    # dominant kernel: gather_accumulate_staged, which takes the first transmissions (a retransmission
    # batch goes to the direct kernel unless it is dense; one that the staged kernel does take adds its
    # time here and not its bytes).  Algorithmic bytes = every packet accepted from a first transmission
    # read once (header + payload + padding = stride) + the accumulator written once per iteration.
    g_ms, g_n = prof["gather"]
    first_accepted = accepted_total - main_leg["resent"]
    g_bytes = first_accepted * L.stride + args.steps * 4 * L.N
    achieved = g_bytes / (g_ms * 1e-3) / 1e9 if g_ms > 0 else 0.0
    ratio_pmc = PMC_TRAFFIC_RATIO.get((_kernel_source_hash(), w.name))
    roofline = dict(bound="hbm", achieved=round(achieved, 1), peak=HBM_PEAK_GBPS, unit="GB/s",
                    frac=round(achieved / HBM_PEAK_GBPS, 4), kernel="gather_accumulate_staged",
                    launches=g_n, avg_launch_ms=round(g_ms / max(g_n, 1), 4),
                    algorithmic_bytes_per_launch=round(g_bytes / max(g_n, 1)),
                    traffic=None if ratio_pmc is None else round(ratio_pmc * g_bytes / max(g_n, 1)))
    # whole-path algorithmic bytes: the gather's (packets read once, accumulator written once).  The
    # mean and the sum of squares are formed in the same pass and the result is left in place, so the
    # compensation pass adds no bytes of its own beyond the spans it zeroes or moves.
    path_bytes = accepted_total * L.stride + args.steps * 4 * L.N
    separate_pass_bytes = path_bytes + args.steps * 8 * L.N     # what a separate read-scale-write finalize pass would add
    acc_info = agg.accumulator_info()
    acc_info.pop("last_pick")
    acc_info["mode"] = args.accumulator
    if trial:
        acc_info["trial"] = trial
    acc_info["copy_per_chunk_step"] = "".join(str(p) for p in picks)

    def leg_summary(leg):
        acc = leg["accepted"]
        return dict(ms_per_step=round(leg["wall"] * 1e3 / leg["steps"], 3), steps=leg["steps"],
                    value=round(acc * 4 * L.P * fill / leg["wall"] / 1e9, 2),
                    packets_per_s=round(acc / leg["wall"], 1),
                    path_hbm_frac=round((acc * L.stride + leg["steps"] * 4 * L.N) / leg["wall"] / 1e9 / HBM_PEAK_GBPS, 4))

    other = {}
    breakdown = None
    if n_extra:
        bounds = {st["it"]: st["bound_ppm"] for st in main_leg["per_step"]}
        leg = run_leg(job, w, extra_its, bounds, profile=True)
        breakdown = dict(steps=n_extra, ms_per_step=round(leg["wall"] * 1e3 / n_extra, 3),
                         **{k: round(v[0] / n_extra, 4) for k, v in leg["prof"].items()})
        other[f"{args.arrivals}+{args.accumulator} (the timed run, its first {n_extra} steps replayed, no event brackets)"] = \
            leg_summary(run_leg(job, w, extra_its, bounds))
        for name in ("queue", "tables"):
            if name != args.arrivals:
                job.queue = form[name]
                other[f"{name}+{args.accumulator}"] = leg_summary(run_leg(job, w, extra_its, bounds))
        job.queue = form[args.arrivals]
        if acc_info["copies"] == 2:
            job.use_single_accumulator()
            run_leg(job, w, extra_its[:1], bounds)          # one untimed step on the new copy
            other[f"{args.arrivals}+one"] = leg_summary(run_leg(job, w, extra_its, bounds))
        elif getattr(job, "plain_agg", None) is not None:
            # the same steps on the context the job started with: one copy, where the library's allocation fell
            job.agg = job.plain_agg
            if job.in_place:
                job.d_out = job.agg.accumulator_tensor(0)
            run_leg(job, w, extra_its[:1], bounds)
            other[f"{args.arrivals}+one"] = leg_summary(run_leg(job, w, extra_its, bounds))

    out = dict(metric="aggregated_gradient_GBps", value=round(value, 2), unit="GB/s", n_gpus=1,
               steps=args.steps, warmup=args.warmup, ms_per_step=round(ms_per_step, 3),
               higher_is_better=True, scaling="weak", vs_baseline=None, dtype="f32", data="synthetic",
               config=dict(workload=f"{w.name}: W={L.W} N={L.N} P={L.P} buckets={L.B} "
                                    f"packets/round={L.W * L.n_pkts} loss={w.loss['kind']} "
                                    f"policy={w.policy['kind']}",
                           placement=job.place, arrival_order=job.order, arrivals=args.arrivals,
                           accumulator=acc_info,
                           result="in place (first accumulator copy)" if job.in_place else "written to a separate buffer",
                           chunk_steps=len(job.chunks), resident_packet_GB=round(job.packets.numel() / 1e9, 2)),
               packets_per_s=round(accepted_total / wall, 1),
               path_hbm_frac=round(path_bytes / wall / 1e9 / HBM_PEAK_GBPS, 4),
               path_hbm_frac_counting_a_separate_finalize_pass=round(separate_pass_bytes / wall / 1e9 / HBM_PEAK_GBPS, 4),
               retransmission_rounds=main_leg["rounds"], resent_packets=main_leg["resent"],
               gpu_event_ms_per_step=round(main_leg["event_ms"] / args.steps, 3),
               kernel_ms_per_step=dict(gather=round(g_ms / args.steps, 4)),
               kernel_ms_per_step_replay_all_groups_bracketed=breakdown,
               sender_side_not_in_value=sender, other_forms=other, per_step=main_leg["per_step"], roofline=roofline)
    if not args.no_cpu_baseline:
        del job
        torch.cuda.empty_cache()
        out["cpu_baseline"] = cpu_baseline(w, max(1_000_000, int(args.cpu_sample_bytes / (4 * L.W))))
    print(json.dumps(out), flush=True)


if __name__ == "__main__":
    main()
