"""Parity at full size, in the configurations bench.py times: the 1.3B-element, W=32 workload with
every packet of a round resident in HBM (167 GB), chunk-streamed application, shuffled placement
and arrival order, burst loss, a 2 % bound with retransmission rounds; and the 124M-element (W=8)
and 355M-element (W=16, 4 KB packets, microburst windows) workloads, each applied as one batch.

Integer outputs are compared in full: the oracle is shown the 8 header bytes of every slot (its
header-only sender and receiver, pinned on the CPU against the payload-carrying ones), the same
masks, arrival orders and retransmission draws, and the whole bitmap, the per-(worker, bucket)
counts and the retransmit list of every probe and the four counters must be equal bit for bit.

The oracle cannot add a whole round's payloads in seconds, so the floats are compared on sampled
buckets (at least 64 plus the first two and the last two): for each it is given exactly that
bucket's packets, in their original relative arrival order, and must reproduce the aggregated
elements of the bucket (aggregation is independent across buckets, so a bucket is an exact
sub-problem), together with the bucket's counts, list entries and bitmap bits once more.  The norm
of the returned gradient is checked against an fp64 reduction of the whole output."""
import dataclasses

import numpy as np
import pytest

import workloads as wl
from harness import record_stat

pytestmark = pytest.mark.gpu


_SURVIVE = {}


def survive(job, rnd):
    if rnd not in _SURVIVE:
        _SURVIVE[rnd] = job.w.survive(0, rnd, job.slot_of)
    return _SURVIVE[rnd]


def bucket_subproblem(job, b, probes, bound_ppm):
    """Run the oracle on bucket b alone; compare with what the GPU reported for it."""
    import oracle
    from harness import FLOAT_TOL
    w, L = job.w, job.L
    s0, s1 = int(L.first_seq[b]), int(L.first_seq[b + 1])
    e0, cnt = int(L.bucket_off[b]), int(L.bucket_cnt[b])
    n = s1 - s0
    ch = next(c for c in job.chunks if c["s0"] <= s0 < c["s1"])
    ci = job.chunks.index(ch)
    # this bucket's packets in their original relative arrival order
    gslots = job.slot_of[:, s0:s1].astype(np.int64)                       # [W, n] global slots
    local = gslots - ch["base"]
    order = wl.arrival_order(job.order, ch["n"], w.seed, ci)
    rank = np.arange(ch["n"], dtype=np.int64)
    if order is not None:
        rank[order.astype(np.int64)] = np.arange(ch["n"])
    by_rank = np.argsort(rank[local.reshape(-1)], kind="stable")          # sub-stream arrival order
    o = oracle.Oracle(L.W, cnt, L.P, [0], [cnt], w.policy.get("eta", 0.5))
    assert o.n_pkts == n
    packets = np.zeros(L.W * n * L.stride, dtype=np.uint8)
    src = np.zeros(L.W * n, dtype=np.uint16)
    grads = []
    for wk in range(L.W):
        g = wl.grad_values(w.seed, wk, 0, e0, cnt, w.sigma_at(0), w.tail_ppm, w.tail_mul)
        grads.append(g)
        o.packetize(wk, job.rnd_id, g, 0, 0, n, packets, src, slot_base=wk * n)   # sub-slot = wk*n + seq
    survive0 = survive(job, 0)[:, s0:s1]
    mask = np.packbits(np.pad(survive0.reshape(-1), (0, (-L.W * n) % 64)), bitorder="little").view(np.uint64)
    o.begin_round(job.rnd_id)
    o.apply_arrivals(packets, src, L.W * n, mask, by_rank.astype(np.uint32))
    rnd = 0
    for pr in probes:
        missing, lst, count, met = o.loss_account(bound_ppm)
        assert np.array_equal(missing[:, 0], pr["missing"][:, b]), f"bucket {b}: missing counts differ at probe {rnd}"
        gl = pr["list"]
        gseq = (gl & np.uint64(0xFFFFFFFF)).astype(np.int64)
        mine = gl[(gseq >= s0) & (gseq < s1)]
        want = (lst & ~np.uint64(0xFFFFFFFF)) | ((lst & np.uint64(0xFFFFFFFF)) + np.uint64(s0))
        assert np.array_equal(mine, want), f"bucket {b}: retransmit entries differ at probe {rnd}"
        if pr["met"]:
            break
        rnd += 1
        if not met:   # resend this bucket's listed packets; the drawn loss of round rnd applies
            ws = (lst >> np.uint64(32)).astype(np.int64)
            ss = (lst & np.uint64(0xFFFFFFFF)).astype(np.int64)
            if rnd in job.d_survive:
                ok = survive(job, rnd)[ws, ss + s0].astype(bool)
                ws, ss = ws[ok], ss[ok]
            o.apply_arrivals(packets, src, L.W * n, None, (ws * n + ss).astype(np.uint32))
    rec = o.received()
    ref = o.finalize()
    got = job.d_out[e0:e0 + cnt].cpu().numpy().astype(np.float64)
    pkt = np.arange(cnt) // L.P
    scale = sum(rec[wk, pkt] * np.abs(grads[wk].astype(np.float64)) for wk in range(L.W)) / L.W
    zero = scale == 0
    assert np.all(got[zero] == 0.0)
    err = np.abs(got - ref)
    rel = (err[~zero] / scale[~zero]).max()
    assert rel <= FLOAT_TOL, f"bucket {b}: float parity {rel:.3e}"
    nz = ref != 0
    plain = err[nz] / np.abs(ref[nz])
    return rec, dict(rel=float(rel), plain_max=float(plain.max()) if nz.any() else 0.0,
                     plain_above=int((plain > FLOAT_TOL).sum()), n=int(cnt))


def integer_outputs_in_full(job, probes, bound_ppm, counters, words):
    """The whole round on the oracle's header-only receiver: every slot's 8 header bytes, the
    chunk steps' masks and arrival orders, then the retransmission batches exactly as
    bench.DeviceJob.step hands them over (every listed packet resent, the drawn loss of the
    round as a mask over the buffer).  Everything integer must be equal in full."""
    import oracle
    w, L = job.w, job.L
    n_slots = L.W * L.n_pkts
    o = oracle.Oracle(L.W, L.N, L.P, L.bucket_off, L.bucket_cnt, w.policy.get("eta", 0.5))
    headers = np.empty(n_slots * 8, dtype=np.uint8)
    src = np.empty(n_slots, dtype=np.uint16)
    for wk in range(L.W):
        o.write_headers(wk, job.rnd_id, 0, L.n_pkts, headers, src, slot_map=job.slot_of[wk])
    o.begin_round(job.rnd_id)
    s0 = survive(job, 0)
    print(f"{w.name}: header-only oracle: {n_slots} headers written", flush=True)
    for ci, ch in enumerate(job.chunks):
        local = (job.slot_of[:, ch["s0"]:ch["s1"]] - np.uint32(ch["base"])).astype(np.uint32)
        mask = wl.slot_mask_words(s0[:, ch["s0"]:ch["s1"]], local)
        order = wl.arrival_order(job.order, ch["n"], w.seed, ci)
        o.apply_arrivals(headers[ch["base"] * 8:], src[ch["base"]:], ch["n"], mask, order, ch["n"],
                         accumulate=False, stride=8)
    for rnd, pr in enumerate(probes):
        print(f"{w.name}: header-only oracle: probe {rnd}", flush=True)
        missing, lst, count, met = o.loss_account(bound_ppm)
        assert count == pr["count"] and met == pr["met"], f"probe {rnd}: list length / all-met differ"
        assert np.array_equal(missing, pr["missing"]), f"probe {rnd}: per-bucket counts differ"
        assert np.array_equal(lst, pr["list"]), f"probe {rnd}: retransmit list differs"
        if met:
            break
        ws = (lst >> np.uint64(32)).astype(np.int64)
        ss = (lst & np.uint64(0xFFFFFFFF)).astype(np.int64)
        slots = job.slot_of[ws, ss].astype(np.uint32)
        mask = wl.slot_mask_words(survive(job, rnd + 1), job.slot_of) if (rnd + 1) in job.d_survive else None
        o.apply_arrivals(headers, src, n_slots, mask, slots, slots.size, accumulate=False, stride=8)
    assert o.counters() == counters, (o.counters(), counters)
    rec = o.received()
    gbits = np.unpackbits(words.view(np.uint8), axis=1, bitorder="little")[:, :L.n_pkts]
    assert np.array_equal(gbits, rec), "bitmap differs"
    assert not np.unpackbits(words.view(np.uint8), axis=1, bitorder="little")[:, L.n_pkts:].any()
    return rec


# workload, bound of the iteration (cfg3: the tight level of its three-level policy; cfg4: its fixed
# bound; cfg5: 2 %), buckets always sampled besides the first two, the last two and seven random ones
FULL_SIZE = [("cfg3", 10_000, ()), ("cfg4", 80_000, ()), ("cfg5", 20_000, (43, 44))]


@pytest.mark.parametrize("name,BOUND_PPM,extra", FULL_SIZE)
def test_full_size_sampled_buckets_and_global_properties(name, BOUND_PPM, extra):
    import torch
    import bench
    w = wl.workload(name)
    mode = bench.default_accumulator(w)
    job = bench.DeviceJob(w, n_masks=1, accumulator=mode)                           # as bench.py runs it:
    if mode == "trial":                                                             # on a caller-owned accumulator
        placed = bench.place_accumulator_by_trial(job, w, n_candidates=2)           # chosen among a few places
        assert placed["adopted"] in [c["where"] for c in placed["candidates"]] and len(placed["candidates"]) == 3
    L = job.L
    probes = []
    res = job.step(0, BOUND_PPM, record=probes)
    counters = job.agg.get_counters()
    # --- properties that hold at any size
    assert counters["stale"] == 0 and counters["invalid"] == 0 and counters["duplicate"] == 0
    assert res["rounds"] >= 1 and probes[-1]["met"] and not probes[0]["met"]
    assert int(probes[-1]["missing"].astype(np.int64).sum()) == L.W * L.n_pkts - counters["accepted"]
    allowed = (BOUND_PPM * L.n_b.astype(np.int64)) // 1_000_000
    assert np.all(probes[-1]["missing"] <= allowed[None, :])            # every bucket meets the bound
    first = probes[0]
    fails = first["missing"] > allowed[None, :]
    assert first["count"] == int(first["missing"][fails].astype(np.int64).sum())
    lst = first["list"]
    assert np.all(lst[1:] > lst[:-1])                                   # sorted, no repeats
    ss = torch.zeros((), dtype=torch.float64, device="cuda")
    for i in range(0, L.N, 1 << 27):
        ss += job.d_out[i:i + (1 << 27)].double().square().sum()
    ref_norm = float(ss.sqrt())
    assert abs(res["norm"] - ref_norm) <= 1e-6 * ref_norm
    # --- sampled buckets against the oracle
    bitmap = torch.empty(L.W * job.agg.words_pw, dtype=torch.int64, device="cuda")
    job.agg.get_bitmap(bitmap)
    words = bitmap.cpu().numpy().view(np.uint64).reshape(L.W, job.agg.words_pw)
    # --- every integer output, in full, against the header-only oracle
    rec_all = integer_outputs_in_full(job, probes, BOUND_PPM, counters, words)
    print(f"{name}: integer outputs equal in full ({len(probes)} probes, {first['count']} list entries)", flush=True)
    # --- floats on sampled buckets: 64 random ones, the first two, the last two, the named extras
    rng = np.random.default_rng(2605)
    pool = np.arange(2, L.B - 2)
    sample = sorted({0, 1, *extra, L.B - 2, L.B - 1, *rng.choice(pool, size=min(64, pool.size), replace=False).tolist()})
    assert len(sample) >= 66
    agg_stats = dict(rel=0.0, plain_max=0.0, plain_above=0, n=0)
    for i, b in enumerate(sample):
        if i % 8 == 0:
            print(f"{name}: sampled bucket {i} of {len(sample)}", flush=True)
        rec, st = bucket_subproblem(job, b, probes, BOUND_PPM)
        s0, s1 = int(L.first_seq[b]), int(L.first_seq[b + 1])
        assert np.array_equal(rec_all[:, s0:s1], rec), f"bucket {b}: bitmap differs"
        agg_stats = dict(rel=max(agg_stats["rel"], st["rel"]), plain_max=max(agg_stats["plain_max"], st["plain_max"]),
                         plain_above=agg_stats["plain_above"] + st["plain_above"], n=agg_stats["n"] + st["n"])
    record_stat(f"{name}_full_size", dict(accumulator=job.agg.accumulator_info(), rounds=res["rounds"], first_list=first["count"],
                                          accepted=counters["accepted"], sampled_buckets=len(sample), rel_to_addends=agg_stats["rel"],
                                          plain_rel_max=agg_stats["plain_max"], plain_rel_above_tol=agg_stats["plain_above"],
                                          n=agg_stats["n"]))
    del rec_all
    # --- the other hand-over form (mask + order + per-slot worker table instead of receive queues)
    # must give the same bits: the sum over workers is formed in worker order either way
    first_out = job.d_out.clone()
    job.queue = False
    job.masks = [job._mask_for(0)]
    res2 = job.step(0, BOUND_PPM)
    assert job.agg.get_counters() == counters and res2["rounds"] == res["rounds"]
    assert res2["norm"] == pytest.approx(res["norm"], rel=1e-12)     # spans may live in other copies this time
    bitmap2 = torch.empty_like(bitmap)
    job.agg.get_bitmap(bitmap2)
    assert torch.equal(bitmap, bitmap2)
    assert torch.equal(first_out.view(torch.int32), job.d_out.view(torch.int32))
    _SURVIVE.clear()
    del job, bitmap, bitmap2, first_out
    torch.cuda.empty_cache()


@pytest.mark.parametrize("rate,fixed_rounds,dblp_rounds", [(0.6, (8, 10), (1, 1)), (0.9, (43, 49), (8, 8))])
def test_microburst_study_rounds_at_model_size_match_the_oracle(rate, fixed_rounds, dblp_rounds):
    """study_microburst.py's figures at the size it runs (EfficientNetB0-sized gradient, 3 workers,
    one accounting unit per worker, whole-iteration burst loss on every retransmission round): the
    number of retransmission rounds and every probe's counts and list, under the fixed tolerance
    and under P_high, must be what the oracle's header-only receiver gets from the same draws."""
    import bench
    import oracle
    w = wl.paper_model_workload("effnetb0", rate, burst_iters=(1,), iterations=3)
    L = w.layout
    job = bench.DeviceJob(w, n_masks=3, per_iteration_retx=True)
    n_slots = L.W * L.n_pkts
    o = oracle.Oracle(L.W, L.N, L.P, L.bucket_off, L.bucket_cnt)
    headers = np.empty(n_slots * 8, dtype=np.uint8)
    src = np.empty(n_slots, dtype=np.uint16)
    for wk in range(L.W):
        o.write_headers(wk, job.rnd_id, 0, L.n_pkts, headers, src, slot_map=job.slot_of[wk])
    order = wl.arrival_order(job.order, n_slots, w.seed, 0)
    seen = {}
    for it, bound in ((0, w.policy["low_ppm"]), (1, w.policy["low_ppm"]), (1, w.policy["high_ppm"]), (2, w.policy["high_ppm"])):
        probes = []
        res = job.step(it, bound, record=probes)
        o.begin_round(job.rnd_id)
        mask = wl.slot_mask_words(w.survive(it, 0, job.slot_of), job.slot_of)
        o.apply_arrivals(headers, src, n_slots, mask, order, n_slots, accumulate=False, stride=8)
        for rnd, pr in enumerate(probes):
            missing, lst, count, met = o.loss_account(bound)
            assert (count, met) == (pr["count"], pr["met"]) and np.array_equal(missing, pr["missing"])
            assert np.array_equal(lst, pr["list"]), f"iteration {it}, probe {rnd}: retransmit list differs"
            if met:
                break
            ok = w.survive(it, rnd + 1, job.slot_of)[(lst >> np.uint64(32)).astype(np.int64),
                                                     (lst & np.uint64(0xFFFFFFFF)).astype(np.int64)].astype(bool)
            slots = job.slot_of[(lst >> np.uint64(32)).astype(np.int64), (lst & np.uint64(0xFFFFFFFF)).astype(np.int64)][ok]
            o.apply_arrivals(headers, src, n_slots, None, slots.astype(np.uint32), slots.size, accumulate=False, stride=8)
        assert o.counters() == job.agg.get_counters()
        assert res["rounds"] == len(probes) - 1
        seen[(it, bound)] = res["rounds"]
    lo, hi = w.policy["low_ppm"], w.policy["high_ppm"]
    assert fixed_rounds[0] <= seen[(1, lo)] <= fixed_rounds[1], seen      # the burst iteration under the fixed tolerance
    assert dblp_rounds[0] <= seen[(1, hi)] <= dblp_rounds[1], seen        # ... and under P_high = p + 40 %
    assert seen[(0, lo)] <= 2 and seen[(2, hi)] == 0, seen                # quiet iterations
    record_stat(f"microburst_rounds_rate_{rate}", dict(rounds={f"{k[0]}@{k[1]}": v for k, v in seen.items()}))
