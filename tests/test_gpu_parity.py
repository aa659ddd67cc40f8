"""GPU parity: the HIP library (through the C-ABI) against the CPU oracle on the same seeded
inputs.  Integer outputs (bitmaps, per-bucket counts, retransmit lists, counters) must be
bit-exact; the fp32 aggregate must be within 1e-5 of the fp64 oracle."""
import dataclasses

import numpy as np
import pytest

import workloads as wl
from harness import (FLOAT_TOL, GpuRx, OracleRx, build_scenario, compare_results, definition_mean,
                     record_stat, run_iteration)

pytestmark = pytest.mark.gpu


def mk(W, sizes, P, loss=0.0, seed=7, place="shuffle", order="shuffle", name="t"):
    off, cnt = wl.buckets_from_sizes(sizes)
    return wl.Workload(name, wl.Layout(W, int(sum(sizes)), P, off, cnt), 1e-3,
                       dict(kind="bernoulli", p=loss) if loss else dict(kind="none"),
                       place, order, dict(kind="fixed", ppm=0), seed=seed)


def both(sc, queue=False, **gpu_kw):
    o, g = OracleRx(sc), GpuRx(sc, queue=queue, **gpu_kw)
    o.packetize_all()
    g.packetize_all()
    return o, g


def run_both(sc, ppm, queue=False, **gpu_kw):
    o, g = both(sc, queue, **gpu_kw)
    ref = run_iteration(o, sc, ppm)
    got = run_iteration(g, sc, ppm)
    return compare_results(got, ref, sc), got, ref


# ------------------------------------------------------------------------------ inputs
def test_device_generator_matches_cpu_generator():
    import torch
    for (w, it, e0, n, tail) in [(0, 0, 0, 1 << 20, 0), (5, 3, 2**33 + 11, 100_003, 10000)]:
        d = torch.empty(n, dtype=torch.float32, device="cuda")
        wl.grad_fill_device(d.data_ptr(), wl.MASTER_SEED, w, it, e0, n, 1e-4, tail, 100.0,
                            torch.cuda.current_stream().cuda_stream)
        torch.cuda.synchronize()
        ref = wl.grad_values(wl.MASTER_SEED, w, it, e0, n, 1e-4, tail, 100.0)
        assert np.array_equal(d.cpu().numpy().view(np.uint32), ref.view(np.uint32))


@pytest.mark.parametrize("W,sizes,P,place", [(2, [1000, 37, 5], 16, "worker_major"), (3, [366 * 70 + 9, 1, 400], 366, "shuffle"),
                                             (4, [5000], 256, "interleave"), (2, [4096 + 17], 1024, "shuffle"), (1, [9], 1, "shuffle")])
def test_packetize_bytes_match_oracle(W, sizes, P, place):
    sc = build_scenario(mk(W, sizes, P, place=place))
    o, g = both(sc)
    assert np.array_equal(g.packets.cpu().numpy(), o.packets)
    assert np.array_equal(g.src.cpu().numpy().view(np.uint16), o.src)


# ------------------------------------------------------------------------------ small / ragged
CASES = [
    # W, bucket sizes, P, loss, bound ppm
    (1, [5], 2, 0.0, 0),
    (2, [3], 2, 0.3, 0),
    (3, [7, 1, 12, 4], 3, 0.3, 100_000),
    (4, [1000, 37, 2048], 16, 0.1, 50_000),
    (5, [70_001, 13, 29_999], 100, 0.05, 20_000),
    (8, [366 * 300 + 5, 1, 366, 365, 367, 50_000], 366, 0.02, 50_000),      # several tiles, ragged tails
    (16, [1024 * 65 + 3, 1023, 1025], 1024, 0.03, 30_000),
    (32, [200_000, 77], 366, 0.05, 10_000),
    (64, [30_000], 50, 0.2, 150_000),
    (7, [256 * 130], 256, 0.01, 0),
    (3, [4_000_000], 1000, 0.01, 8_000),                                     # one bucket = whole-round accounting
    (2, [65535 * 3 + 1], 65535, 0.0, 0),                                     # maximum packet length
    (4, [600 * 40 + 7, 100], 600, 0.05, 30_000),                             # three 1 KB passes per packet
    (3, [1400 * 33 + 5], 1400, 0.05, 30_000),                                # six passes: generic staged path
    (2, [3000 * 9 + 1], 3000, 0.1, 50_000),                                  # 12 KB packets: two-packet groups
    (2, [4000 * 5 + 3], 4000, 0.1, 50_000),                                  # too long to stage: direct stores
]


@pytest.mark.parametrize("W,sizes,P,loss,ppm", CASES)
def test_parity_small_and_ragged(W, sizes, P, loss, ppm):
    stats, got, ref = run_both(build_scenario(mk(W, sizes, P, loss)), ppm)
    assert stats["rel_to_addends"] <= FLOAT_TOL


@pytest.mark.parametrize("W,sizes,P,loss,ppm", CASES)
def test_parity_small_and_ragged_receive_queue(W, sizes, P, loss, ppm):
    """The same cases with every batch handed over as a receive queue of descriptors."""
    stats, got, ref = run_both(build_scenario(mk(W, sizes, P, loss)), ppm, queue=True)
    assert stats["rel_to_addends"] <= FLOAT_TOL


@pytest.mark.parametrize("result", ["in_place", "caller"])
@pytest.mark.parametrize("W,sizes,P,loss,ppm", [c for c in CASES if c[0] & (c[0] - 1) == 0])
def test_parity_small_and_ragged_in_place(W, sizes, P, loss, ppm, result):
    """The in-place forms of finalize (power-of-two W): the result is read from the library's first
    accumulator copy, or the accumulator is a buffer of the caller's that is also given as d_out.
    Same bits as the copying form."""
    sc = build_scenario(mk(W, sizes, P, loss))
    stats, got, ref = run_both(sc, ppm, queue=(result == "caller"), result=result)
    assert stats["rel_to_addends"] <= FLOAT_TOL
    g1 = GpuRx(sc); g1.packetize_all()
    one = run_iteration(g1, sc, ppm)
    assert np.array_equal(one["out"].view(np.uint32), got["out"].view(np.uint32))
    assert one["norm"] == got["norm"] and one["counters"] == got["counters"]


# ------------------------------------------------------------------------------ two accumulator copies
TWO_COPY_CASES = [CASES[i] for i in (3, 5, 6, 7, 10, 13, 14, 15)]


@pytest.mark.parametrize("result", ["copy", "in_place", "caller"])
@pytest.mark.parametrize("policy", [2, 3])      # always the second copy; alternate per batch
@pytest.mark.parametrize("W,sizes,P,loss,ppm", TWO_COPY_CASES)
def test_two_accumulator_copies_give_the_same_bits(W, sizes, P, loss, ppm, policy, result):
    """Where a span lives must not show in any result: first transmissions and retransmission
    rounds land in different copies under these policies; the in-place forms of finalize move
    the spans of the second copy into the first."""
    if result != "copy" and W & (W - 1):
        pytest.skip("the in-place form needs a power-of-two worker count")
    sc = build_scenario(mk(W, sizes, P, loss))
    stats, got, ref = run_both(sc, ppm, acc_copies=2, acc_policy=policy, result=result)
    assert stats["rel_to_addends"] <= FLOAT_TOL
    g1 = GpuRx(sc); g1.packetize_all()
    one = run_iteration(g1, sc, ppm)
    assert np.array_equal(one["out"].view(np.uint32), got["out"].view(np.uint32))
    assert one["norm"] == got["norm"] and one["counters"] == got["counters"]


@pytest.mark.parametrize("queue", [False, True])
def test_batches_alternate_between_accumulator_copies(queue):
    """Four batches over the same spans, new spans going to alternating copies: every later batch
    must find and update a span in the copy that holds it."""
    sc = build_scenario(mk(5, [366 * 120 + 11, 3000, 1], 366, 0.1, place="shuffle", order="shuffle"))
    L = sc.L
    n = L.W * L.n_pkts
    part = np.random.default_rng(11).integers(0, 4, size=n)
    o, g = both(sc, queue, acc_copies=2, acc_policy=3)
    assert g.agg.accumulator_info()["copies"] == 2
    picks = []
    for rx in (o, g):
        rx.begin_round(sc.rnd_id)
        for k in range(4):
            rx.apply(0, n, sc.batches[0].mask, np.flatnonzero(part == k).astype(np.uint32))
            if rx is g:
                picks.append(g.agg.accumulator_info()["last_pick"])
    assert picks == [0, 1, 0, 1]
    assert np.array_equal(g.bitmap(), o.bitmap()) and g.counters() == o.counters()
    from harness import abs_scale
    ref, got = o.finalize(), g.finalize().astype(np.float64)
    scale = abs_scale(sc, sc.survive0)
    nz = scale > 0
    assert (np.abs(got - ref)[nz] / scale[nz]).max() <= FLOAT_TOL and np.all(got[~nz] == 0)
    assert g.phase_signal()[0] == pytest.approx(o.phase_signal()[0], rel=1e-6)


@pytest.mark.parametrize("place", [0, 1])
def test_automatic_copy_choice_on_a_buffer_large_enough_to_be_measured(place):
    """1.3 GB of packets: under the automatic policy the library times its probe kernel on the
    buffer before the first batch (place 0: against two plain copies; place 1: against the copy
    the bounded search found, if it found one).  Whatever it decides, the bits are those of a
    one-copy run."""
    sc = build_scenario(mk(8, [20_000_000, 15_000_000, 5_000_007], 366, 0.03, place="shuffle", order="shuffle"))
    g1 = GpuRx(sc, queue=True); g1.packetize_all()
    one = run_iteration(g1, sc, 20_000)
    del g1
    g2 = GpuRx(sc, queue=True, acc_copies=2, acc_policy=0, acc_place=place); g2.packetize_all()
    two = run_iteration(g2, sc, 20_000)
    info = g2.agg.accumulator_info()
    print("accumulator after the run:", info)
    assert info["copies"] == (2 if place == 0 else info["copies"])
    assert np.array_equal(one["out"].view(np.uint32), two["out"].view(np.uint32))
    assert one["counters"] == two["counters"] and one["rounds"] == two["rounds"]
    assert two["norm"] == pytest.approx(one["norm"], rel=1e-12)
    for a, b in zip(one["probes"], two["probes"]):
        assert np.array_equal(a["missing"], b["missing"]) and np.array_equal(a["list"], b["list"])


def test_accumulator_api():
    from paper_2605_01989_amd import DblpError, binding
    sc = build_scenario(mk(2, [1000], 10))
    g = GpuRx(sc)
    info = g.agg.accumulator_info()
    assert (info["copies"], info["distinct_thirds"], info["last_pick"]) == (1, False, 0)
    g.begin_round(1)
    g.agg.accumulator_copies(2)                           # discards the round in progress
    with pytest.raises(DblpError) as e:
        g.apply(0, 200, None, None)
    assert e.value.code == binding.ESTATE
    for bad in (0, 3):
        with pytest.raises(DblpError) as e:
            g.agg.accumulator_copies(bad)
        assert e.value.code == binding.EINVAL
    with pytest.raises(DblpError) as e:
        g.agg.accumulator_policy(4)
    assert e.value.code == binding.EINVAL
    with pytest.raises(DblpError) as e:
        g.agg.accumulator_copies(2, place=2)              # only 0 (plain) and 1 (bounded search) exist
    assert e.value.code == binding.EINVAL
    g.agg.accumulator_copies(1)
    assert g.agg.accumulator_info()["copies"] == 1
    with pytest.raises(DblpError) as e:
        g.agg.accumulator_ptr(1)
    assert e.value.code == binding.EINVAL
    assert g.agg.accumulator_ptr(0) != 0


def test_accumulator_modes_of_the_configuration():
    """dblp_config.accumulator_mode: single (nothing measured), pair (plain second copy), search
    (bounded: here a twentieth of the free memory and one second, so it may well find nothing and
    must then run with one copy); caller-owned buffers; the combinations that are refused."""
    import torch
    import paper_2605_01989_amd as dblp
    from paper_2605_01989_amd import DblpError, binding
    sc = build_scenario(mk(4, [366 * 50 + 3, 900], 366, 0.1))
    L = sc.L
    mk_agg = lambda **kw: dblp.Aggregator(L.W, L.N, L.P, L.bucket_off, L.bucket_cnt, **kw)
    a = mk_agg()
    assert a.accumulator_info()["copies"] == 1 and a.accumulator_info()["placement_steps"] == 0
    b = mk_agg(accumulator_mode=binding.ACCMODE_PAIR)
    assert b.accumulator_info()["copies"] == 2 and b.accumulator_ptr(1) != b.accumulator_ptr(0)
    free0 = torch.cuda.mem_get_info()[0]
    c = mk_agg(accumulator_mode=binding.ACCMODE_SEARCH, search_free_fraction=0.05, search_seconds=1.0)
    info = c.accumulator_info()
    assert info["copies"] in (1, 2) and info["placement_seconds"] < 3.0
    assert torch.cuda.mem_get_info()[0] > free0 - (1 << 30)      # the search released what it held
    buf = [torch.empty(L.N, dtype=torch.float32, device="cuda") for _ in range(2)]
    d = mk_agg(d_accumulator=(buf[0], None))
    assert d.accumulator_ptr(0) == buf[0].data_ptr()
    with pytest.raises(DblpError) as e:
        d.accumulator_copies(2)                           # the accumulator is the caller's
    assert e.value.code == binding.EINVAL
    e2 = mk_agg(accumulator_mode=binding.ACCMODE_PAIR, d_accumulator=(buf[0], buf[1]))
    assert e2.accumulator_info()["copies"] == 2 and e2.accumulator_ptr(1) == buf[1].data_ptr()
    for bad in (dict(accumulator_mode=3), dict(accumulator_mode=binding.ACCMODE_SEARCH, d_accumulator=(buf[0], None)),
                dict(d_accumulator=(buf[0], buf[1])), dict(accumulator_mode=binding.ACCMODE_PAIR, d_accumulator=(buf[0], buf[0])),
                dict(accumulator_mode=binding.ACCMODE_PAIR, d_accumulator=(buf[0], None)),
                dict(d_accumulator=(buf[0][1:], None)), dict(search_free_fraction=0.95), dict(search_seconds=-1.0)):
        with pytest.raises(DblpError) as e:
            mk_agg(**bad)
        assert e.value.code == binding.EINVAL, bad
    # every mode gives the bits of the single-copy run
    g1 = GpuRx(sc); g1.packetize_all()
    one = run_iteration(g1, sc, 20_000)
    for agg in (b, c, d, e2):
        g = GpuRx(sc)
        g.agg = agg
        if agg in (d, e2):
            g.d_out, g.result = buf[0], "caller"
        g.packetize_all()
        got = run_iteration(g, sc, 20_000)
        assert np.array_equal(one["out"].view(np.uint32), got["out"].view(np.uint32)) and one["norm"] == got["norm"]


def test_in_place_finalize_needs_a_power_of_two_worker_count_and_survives_later_arrivals():
    from paper_2605_01989_amd import DblpError, binding
    sc = build_scenario(mk(3, [500], 10))
    g = GpuRx(sc, result="in_place"); g.packetize_all()
    g.begin_round(sc.rnd_id)
    g.apply(0, 150, None, None)
    with pytest.raises(DblpError) as e:
        g.finalize()
    assert e.value.code == binding.EINVAL
    # W = 4, two copies, alternating: finalize in place in the middle of the round (spans move to
    # copy 0, missing spans are zeroed), then the rest arrives and finalize runs again
    sc = build_scenario(mk(4, [366 * 90 + 11, 2000], 366, 0.1, place="shuffle", order="shuffle"))
    L = sc.L
    n = L.W * L.n_pkts
    part = np.random.default_rng(3).integers(0, 3, size=n)
    o, g = both(sc, acc_copies=2, acc_policy=3, result="in_place")
    for rx in (o, g):
        rx.begin_round(sc.rnd_id)
        for k in range(3):
            rx.apply(0, n, sc.batches[0].mask, np.flatnonzero(part == k).astype(np.uint32))
            out = rx.finalize()
            sig = rx.phase_signal() if k == 2 else None
        rx.last = (out, sig)
    from harness import abs_scale
    ref, got = o.last[0], g.last[0].astype(np.float64)
    scale = abs_scale(sc, sc.survive0)
    nz = scale > 0
    assert (np.abs(got - ref)[nz] / scale[nz]).max() <= FLOAT_TOL and np.all(got[~nz] == 0)
    assert g.last[1][0] == pytest.approx(o.last[1][0], rel=1e-6)
    assert np.array_equal(g.bitmap(), o.bitmap()) and g.counters() == o.counters()


@pytest.mark.parametrize("queue", [False, True])
def test_more_buckets_than_the_on_chip_table_holds(queue):
    """5000 small buckets: the bucket boundaries no longer fit the index kernel's on-chip copy
    and are searched in device memory."""
    rng = np.random.default_rng(5)
    sizes = [int(x) for x in rng.integers(1, 40, size=5000)]
    stats, got, ref = run_both(build_scenario(mk(3, sizes, 7, 0.1)), 100_000, queue=queue)
    assert stats["rel_to_addends"] <= FLOAT_TOL


@pytest.mark.parametrize("place,order", [("worker_major", "identity"), ("worker_major", "reverse"),
                                         ("interleave", "identity"), ("shuffle", "shuffle")])
def test_result_is_bitwise_independent_of_arrival_permutation(place, order):
    base = mk(8, [366 * 200 + 7, 5000], 366, 0.05, place="worker_major", order="identity")
    sc0 = build_scenario(base)
    g0 = GpuRx(sc0); g0.packetize_all()
    r0 = run_iteration(g0, sc0, 20_000)
    sc1 = build_scenario(base, place=place, order=order)
    g1 = GpuRx(sc1); g1.packetize_all()
    r1 = run_iteration(g1, sc1, 20_000)
    assert np.array_equal(r0["out"].view(np.uint32), r1["out"].view(np.uint32))
    assert np.array_equal(r0["bitmap"], r1["bitmap"]) and r0["norm"] == r1["norm"]
    assert all(np.array_equal(a["list"], b["list"]) for a, b in zip(r0["probes"], r1["probes"]))


def test_zero_loss_equals_fp32_sequential_mean_exactly():
    """No loss: the GPU sums workers in index order in fp32 and scales by 1/W (W a power of two)."""
    sc = build_scenario(mk(4, [100_000, 333], 366))
    g = GpuRx(sc); g.packetize_all()
    res = run_iteration(g, sc, 0)
    s = sc.grad(0).copy()
    for w in range(1, 4):
        s = (s + sc.grad(w)).astype(np.float32)
    assert np.array_equal(res["out"], s * np.float32(0.25))
    assert res["rounds"] == 0 and res["probes"][0]["met"]


@pytest.mark.parametrize("queue", [False, True])
def test_multiple_batches_accumulate_into_existing_spans(queue):
    """Arrivals delivered in three separate batches, workers interleaved: later batches add to
    spans that earlier batches wrote (read-modify-write path) and never double count."""
    sc = build_scenario(mk(6, [366 * 90 + 11, 2000], 366, 0.1, place="worker_major", order="identity"))
    L = sc.L
    n = L.W * L.n_pkts
    rng = np.random.default_rng(3)
    part = rng.integers(0, 3, size=n)
    o, g = both(sc, queue)
    for rx in (o, g):
        rx.begin_round(sc.rnd_id)
        for k in range(3):
            order = np.flatnonzero(part == k).astype(np.uint32)
            rx.apply(0, n, sc.batches[0].mask, order)
        rx.apply(0, n, sc.batches[0].mask, None)   # everything again: all duplicates
    assert np.array_equal(g.bitmap(), o.bitmap()) and np.array_equal(o.bitmap(), sc.survive0)
    assert g.counters() == o.counters()
    assert o.counters()["duplicate"] == int(sc.survive0.sum())
    ref, got = o.finalize(), g.finalize().astype(np.float64)
    assert np.allclose(ref, definition_mean(sc, sc.survive0), rtol=1e-14, atol=0)
    from harness import abs_scale
    scale = abs_scale(sc, sc.survive0)
    nz = scale > 0
    assert (np.abs(got - ref)[nz] / scale[nz]).max() <= FLOAT_TOL and np.all(got[~nz] == 0)


def test_a_round_recorded_under_stream_capture_replays_to_the_eager_result():
    """begin_round, the batches of a round and finalize only launch kernels on the context's stream,
    so a caller may record them into a graph: three replays, with eager work of the program between
    them, each give the bits and the counters of the eager run."""
    import torch
    sc = build_scenario(mk(8, [366 * 300 + 5, 4000, 77], 366, 0.05))
    L = sc.L
    eager = GpuRx(sc); eager.packetize_all()
    eager.begin_round(sc.rnd_id)
    for b in sc.batches:
        eager.apply(b.slot_base, b.n_slots, b.mask, b.order)
    want = eager.finalize().copy()
    want_norm, want_counters, want_bitmap = eager.phase_signal()[0], eager.counters(), eager.bitmap()
    side = torch.cuda.Stream()
    with torch.cuda.stream(side):
        g = GpuRx(sc)                      # its context takes the current stream: the side stream
        g.packetize_all()
        st = g.agg.stride
        dev = [(b, None if b.mask is None else torch.from_numpy(b.mask.view(np.int64)).cuda(),
                None if b.order is None else torch.from_numpy(np.asarray(b.order, dtype=np.uint32).view(np.int32)).cuda())
               for b in sc.batches]
        side.synchronize()
        graph = torch.cuda.CUDAGraph()
        with torch.cuda.graph(graph, stream=side):
            g.agg.begin_round(sc.rnd_id)
            for b, d_mask, d_order in dev:
                g.agg.apply_arrivals(g.packets[b.slot_base * st:], g.src[b.slot_base:], b.n_slots, d_mask, d_order,
                                     b.n_slots if d_order is None else d_order.numel())
            g.agg.finalize(g.d_out)
        for rep in range(3):
            g.d_out.fill_(7.0)             # eager work between the replays
            torch.cuda.synchronize()
            graph.replay()
            side.synchronize()
            got = g.d_out.cpu().numpy()
            assert np.array_equal(got.view(np.uint32), want.view(np.uint32)), f"replay {rep}"
            assert g.phase_signal()[0] == want_norm and g.counters() == want_counters, f"replay {rep}"
            assert np.array_equal(g.bitmap(), want_bitmap), f"replay {rep}"
            g.agg.set_prev_norm(None)


@pytest.mark.parametrize("W,n_elems", [(2, 1_200_000), (20, 120_000)])
def test_small_batches_scattered_over_a_long_round(W, n_elems):
    """A dense first batch, then batches of a handful of packets scattered over a round of up to 1.2 M
    sequence numbers (the direct gather looks through the arrival index of many groups at once and
    walks the few that hold an entry: more than 64 groups per block at the larger size), a batch that
    fills a contiguous run, and one that is mostly copies of delivered packets."""
    sc = build_scenario(mk(W, [n_elems, 37], 1, place="worker_major", order="identity"))
    L = sc.L
    n = L.W * L.n_pkts
    rng = np.random.default_rng(11)
    run = np.arange(5000, 5300, dtype=np.int64)                        # 300 consecutive packets of worker 0
    held = np.unique(np.concatenate([rng.choice(n, size=1700, replace=False), run]))
    first = np.setdiff1d(np.arange(n, dtype=np.int64), held)
    scattered = rng.choice(np.setdiff1d(held, run), size=40, replace=False)
    batches = [rng.permutation(first), scattered[:12], run, scattered[12:28],
               np.concatenate([rng.choice(first, size=50, replace=False), scattered[28:33]])]
    o, g = both(sc)
    for rx in (o, g):
        rx.begin_round(sc.rnd_id)
        for b in batches:
            rx.apply(0, n, None, b.astype(np.uint32))
    delivered = np.ones(n, dtype=bool)
    delivered[np.setdiff1d(held, np.concatenate([run, scattered[:33]]))] = False
    assert np.array_equal(o.bitmap().reshape(-1).astype(bool), delivered)
    assert np.array_equal(g.bitmap(), o.bitmap())
    assert g.counters() == o.counters() and o.counters()["duplicate"] == 50
    m_o, l_o, c_o, met_o = o.loss_account(0)
    m_g, l_g, c_g, met_g = g.loss_account(0)
    assert c_g == c_o == int((~delivered).sum()) and np.array_equal(m_g, m_o) and np.array_equal(l_g[:c_g], l_o[:c_o])
    ref, got = o.finalize(), g.finalize().astype(np.float64)
    from harness import abs_scale
    scale = abs_scale(sc, delivered.reshape(L.W, L.n_pkts).astype(np.uint8))
    nz = scale > 0
    assert (np.abs(got - ref)[nz] / scale[nz]).max() <= FLOAT_TOL and np.all(got[~nz] == 0)
    assert abs(g.phase_signal()[0] - o.phase_signal()[0]) <= 1e-6 * o.phase_signal()[0] + 2.0 ** -22 * np.sqrt((scale ** 2).sum())


@pytest.mark.parametrize("queue", [False, True])
def test_stale_duplicate_and_invalid_packets(queue):
    sc = build_scenario(mk(2, [100, 7], 10, place="worker_major", order="identity"))
    o, g = both(sc, queue)
    p = o.packets.reshape(-1, sc.L.stride)
    p[0, 0:4] = np.frombuffer(np.uint32(11).tobytes(), np.uint8)        # seq out of range
    p[1, 6:8] = np.frombuffer(np.uint16(9).tobytes(), np.uint8)         # wrong length
    p[10, 6:8] = np.frombuffer(np.uint16(10).tobytes(), np.uint8)       # tail packet claiming full length
    p[3, 4:6] = np.frombuffer(np.uint16(sc.rnd_id - 1).tobytes(), np.uint8)   # previous round
    o.src[2] = 2                                                        # worker out of range
    g.upload_packets(o.packets, o.src)
    order = np.concatenate([np.arange(22), [22, 1000], [5, 5, 6]]).astype(np.uint32)
    for rx in (o, g):
        rx.begin_round(sc.rnd_id)
        rx.apply(0, 22, None, order)
    assert o.counters() == dict(accepted=17, duplicate=3, stale=1, invalid=6)
    assert g.counters() == o.counters()
    assert np.array_equal(g.bitmap(), o.bitmap())
    assert np.allclose(g.finalize(), o.finalize(), rtol=1e-6, atol=0)


@pytest.mark.parametrize("queue", [False, True])
def test_first_arrival_of_conflicting_copies_wins(queue):
    """Two slots claim the same (worker, seq) with different payloads: the earlier arrival is used."""
    sc = build_scenario(mk(1, [40], 10, place="worker_major", order="identity"))
    o, g = both(sc, queue)
    p = o.packets.reshape(-1, sc.L.stride)
    p[3, :8] = p[2, :8]                     # slot 3 now also claims seq 2 (with seq 3's payload)
    g.upload_packets(o.packets, o.src)
    for order in ([0, 1, 2, 3], [0, 1, 3, 2], [3, 2, 1, 0]):
        for rx in (o, g):
            rx.begin_round(sc.rnd_id)
            rx.apply(0, 4, None, np.array(order, dtype=np.uint32))
        assert g.counters() == o.counters() == dict(accepted=3, duplicate=1, stale=0, invalid=0)
        assert np.array_equal(g.finalize().astype(np.float64), o.finalize())


def test_whole_round_stale_leaves_everything_zero():
    sc = build_scenario(mk(3, [5000], 64))
    o, g = OracleRx(sc), GpuRx(sc)
    o.packetize_all(rnd_id=sc.rnd_id + 1)
    g.packetize_all(rnd_id=sc.rnd_id + 1)
    ref = run_iteration_noloop(o, sc)
    got = run_iteration_noloop(g, sc)
    assert got["counters"] == ref["counters"] and ref["counters"]["stale"] == 3 * sc.L.n_pkts
    assert not got["out"].any() and not got["bitmap"].any() and got["norm"] == 0.0


def run_iteration_noloop(rx, sc):
    rx.begin_round(sc.rnd_id)
    for b in sc.batches:
        rx.apply(b.slot_base, b.n_slots, b.mask, b.order)
    out = rx.finalize()
    norm, delta, crit = rx.phase_signal()
    return dict(out=out, norm=norm, bitmap=rx.bitmap(), counters=rx.counters())


# ------------------------------------------------------------------------------ probe edge cases
def test_bound_extremes_and_list_capacity():
    sc = build_scenario(mk(4, [64 * 50] * 5, 50, 0.2))
    o, g = both(sc)
    for rx in (o, g):
        rx.begin_round(sc.rnd_id)
        b = sc.batches[0]
        rx.apply(0, b.n_slots, b.mask, b.order)
    for ppm in (0, 1_000_000, 200_000, 250_000):
        mo, lo, co, meto = o.loss_account(ppm)
        mg, lg, cg, metg = g.loss_account(ppm)
        assert np.array_equal(mo, mg) and np.array_equal(lo, lg) and (co, meto) == (cg, metg)
    mo, lo, co, _ = o.loss_account(0)
    assert co == int((1 - sc.survive0).sum())
    mg, lg, cg, metg = g.loss_account(0, capacity=10)       # truncated list
    assert cg == co and not metg and np.array_equal(lg, lo[:10])
    count, met, trunc = g.agg.loss_account(0, None, None, 0)
    assert trunc and count == co


def test_empty_batch_and_nothing_received():
    sc = build_scenario(mk(2, [1000], 10))
    o, g = both(sc)
    for rx in (o, g):
        rx.begin_round(sc.rnd_id)
        rx.apply(0, 200, None, np.zeros(0, dtype=np.uint32), 0)
    assert g.counters() == o.counters() == dict(accepted=0, duplicate=0, stale=0, invalid=0)
    mo, lo, co, meto = o.loss_account(0)
    mg, lg, cg, metg = g.loss_account(0)
    assert np.array_equal(mo, mg) and np.array_equal(lo, lg) and co == cg == 200
    assert not g.finalize().any()
    assert g.phase_signal()[0] == 0.0


def test_receive_queue_descriptor_fields():
    """Reserved bits, a worker or a slot out of range make a descriptor invalid; nothing else of
    the batch is disturbed."""
    import torch
    from paper_2605_01989_amd import DblpError, binding
    sc = build_scenario(mk(2, [100], 10, place="worker_major", order="identity"))
    o, g = both(sc, queue=True)
    q = np.arange(20, dtype=np.uint64) | (np.repeat(np.arange(2, dtype=np.uint64), 10) << np.uint64(32))
    bad = np.array([q[4] | np.uint64(1) << np.uint64(48),      # reserved bit
                    np.uint64(5) | np.uint64(2) << np.uint64(32),      # worker 2 of 2
                    np.uint64(20) | np.uint64(1) << np.uint64(32),     # slot 20 of 20
                    q[7]], dtype=np.uint64)                            # a plain duplicate
    d_q = torch.from_numpy(np.concatenate([q, bad]).view(np.int64)).cuda()
    g.begin_round(sc.rnd_id)
    g.agg.apply_arrivals_queue(g.packets, 20, d_q)
    assert g.counters() == dict(accepted=20, duplicate=1, stale=0, invalid=3)
    o.begin_round(sc.rnd_id)
    o.apply(0, 20, None, None)
    assert np.array_equal(g.bitmap(), o.bitmap())
    assert np.array_equal(g.finalize().astype(np.float64), o.finalize().astype(np.float32).astype(np.float64))
    with pytest.raises(DblpError) as e:
        g.agg.apply_arrivals_queue(g.packets, 20, None, 5)
    assert e.value.code == binding.EINVAL
    with pytest.raises(DblpError) as e:
        g.agg.apply_arrivals_queue(g.packets, 20, d_q.view(torch.int32)[1:], 5)     # misaligned queue
    assert e.value.code == binding.EINVAL


def test_api_errors():
    import torch
    from paper_2605_01989_amd import DblpError, binding
    import paper_2605_01989_amd as dblp
    sc = build_scenario(mk(2, [1000], 10))
    g = GpuRx(sc)
    with pytest.raises(DblpError) as e:
        g.apply(0, 200, None, None)                       # before begin_round
    assert e.value.code == binding.ESTATE
    g.begin_round(1)
    with pytest.raises(DblpError) as e:
        g.agg.phase_signal()                              # no finalize yet
    assert e.value.code == binding.ESTATE
    with pytest.raises(DblpError) as e:
        g.agg.finalize(g.d_out, compensation=1)
    assert e.value.code == binding.EINVAL
    with pytest.raises(DblpError) as e:
        g.agg.apply_arrivals(g.packets[8:], g.src, 10)    # misaligned packet buffer
    assert e.value.code == binding.EINVAL
    with pytest.raises(DblpError) as e:
        g.agg.loss_account(1_000_001, g.d_missing, g.d_list)
    assert e.value.code == binding.EINVAL
    grad = torch.zeros(500, device="cuda")
    with pytest.raises(DblpError) as e:                   # packets reach beyond the gradient window
        g.agg.packetize(0, 1, grad, 0, 0, 100, g.packets, g.src)
    assert e.value.code == binding.EINVAL
    bad_map = torch.full((50,), 10_000, dtype=torch.int32, device="cuda")
    with pytest.raises(DblpError) as e:                   # slot map points outside the buffer
        g.agg.packetize(0, 1, grad, 0, 0, 50, g.packets, g.src, d_slot_map=bad_map)
    assert e.value.code == binding.EINVAL
    for bad in (dict(n_workers=0), dict(n_workers=65), dict(payload_floats=0), dict(bucket_cnt=[999])):
        kw = dict(n_workers=2, n_elems=1000, payload_floats=10, bucket_off=[0], bucket_cnt=[1000])
        kw.update(bad)
        with pytest.raises(DblpError):
            dblp.Aggregator(**kw)


# ------------------------------------------------------------------------------ phase signal
def test_phase_signal_on_a_vector_and_truth_table():
    import torch
    sc = build_scenario(mk(2, [100_003], 100))
    g = GpuRx(sc)
    g.begin_round(1)
    v = torch.from_numpy(sc.grad(0)).cuda()
    ref = float(np.sqrt((sc.grad(0).astype(np.float64) ** 2).sum()))
    norm, delta, crit = g.agg.phase_signal(v)
    assert abs(norm - ref) <= 1e-6 * ref and crit and np.isinf(delta)
    for prev_mul, want in [(2.0, True), (1.0 / 1.5, True), (1.0 / 0.51, False), (1.0, False)]:
        g.agg.set_prev_norm(norm * prev_mul)
        n2, d2, c2 = g.agg.phase_signal(v)
        assert n2 == norm and c2 == want and abs(d2 - abs(prev_mul - 1) / prev_mul) < 1e-9
    assert g.agg.get_prev_norm() == norm


# ------------------------------------------------------------------------------ named workloads
def test_cfg1_full():
    stats, got, ref = run_both(build_scenario(wl.workload("cfg1")), 50_000)
    assert ref["counters"]["accepted"] >= int(0.985 * 16384)
    record_stat("cfg1_full", dict(rounds=ref["rounds"], first_list=ref["probes"][0]["count"], **stats))


def test_cfg2_full():
    stats, got, ref = run_both(build_scenario(wl.workload("cfg2")), 50_000)
    record_stat("cfg2_full", dict(rounds=ref["rounds"], first_list=ref["probes"][0]["count"], **stats))


def test_cfg3_schedule_scaled_down():
    """GPT-2-small tensor table scaled to 6M elements, Gilbert-Elliott loss, 15 iterations of the
    three-level policy driven by the phase signal.  The bound fed to both sides comes from the
    oracle's signal; the GPU's signal must map to the same bound."""
    import oracle as orc
    import paper_2605_01989_amd as dblp
    w = wl.scaled_down(wl.workload("cfg3"), 6_000_000)
    w = dataclasses.replace(w, scale_schedule=tuple(w.scale_schedule[8:23]), iterations=15)
    pol = w.policy
    bound = pol["ppm"][0]                         # first iteration: tight
    prev_o = prev_g = None
    seen = set()
    for it in range(w.iterations):
        sc = build_scenario(w, it)
        o, g = both(sc)
        o.o.set_prev_norm(prev_o)
        g.agg.set_prev_norm(prev_g)
        ref = run_iteration(o, sc, bound)
        got = run_iteration(g, sc, bound)
        compare_results(got, ref, sc)
        prev_o, prev_g = ref["norm"], got["norm"]
        nb_o = orc.policy_three_level(ref["rel_delta"], pol["eta"], *pol["ppm"])
        nb_g = dblp.policy_three_level(got["rel_delta"], pol["eta"], *pol["ppm"])
        assert nb_o == nb_g
        seen.add(bound)
        bound = nb_o
    assert seen == set(pol["ppm"]), seen          # the schedule visits all three levels


def test_cfg4_microburst_scaled_down():
    w = wl.scaled_down(wl.workload("cfg4"), 20_000_000)
    stats, got, ref = run_both(build_scenario(w), 80_000)
    assert ref["rounds"] >= 1
    record_stat("cfg4_scaled_down", dict(rounds=ref["rounds"], first_list=ref["probes"][0]["count"], **stats))


def test_cfg5_chunked_scaled_down():
    """Chunk-streamed application (44 buckets per step), W=32, heavy-tailed values, burst loss."""
    w = wl.workload("cfg5")
    L = w.layout
    off, cnt = wl.buckets_fixed(4_000_000, L.P, 64)
    w = dataclasses.replace(w, layout=wl.Layout(L.W, 4_000_000, L.P, off, cnt))
    sc = build_scenario(w)
    assert len(sc.batches) == 4
    stats, got, ref = run_both(sc, 20_000)
    assert ref["rounds"] >= 1
    record_stat("cfg5_chunked_scaled_down", dict(rounds=ref["rounds"], first_list=ref["probes"][0]["count"], **stats))


def test_cfg5_schedule_scaled_down():
    """The 1.3B-element recipe (W=32, 44-bucket chunk steps, Gilbert-Elliott loss at 5x rate, 1 %
    heavy-tail entries) on 4M elements: 12 iterations of the continuous 2-15 % policy driven by the
    phase signal (Eq. 1; Alg. Server, tolerance block), over the stretch of its gradient-scale
    schedule that holds the x0.45 drop, plus one x0.75 step so that a bound in the middle of the
    range occurs.  The bound fed to both sides comes from the oracle's signal; the GPU's signal
    must map to the same 1000-ppm step every iteration."""
    import oracle as orc
    import paper_2605_01989_amd as dblp
    w = wl.workload("cfg5")
    L = w.layout
    off, cnt = wl.buckets_fixed(4_000_000, L.P, 64)
    sched = list(w.scale_schedule[6:16])
    sched += [sched[-1] * 0.75, sched[-1] * 0.75 * 0.97]
    w = dataclasses.replace(w, layout=wl.Layout(L.W, 4_000_000, L.P, off, cnt), scale_schedule=tuple(sched),
                            iterations=len(sched))
    pol = w.policy
    assert pol["kind"] == "linear" and (pol["lo_ppm"], pol["hi_ppm"]) == (20_000, 150_000)
    bound = pol["lo_ppm"]                         # first iteration: critical, tightest bound
    prev_o = prev_g = None
    seen, rounds = [], []
    for it in range(w.iterations):
        sc = build_scenario(w, it)
        assert len(sc.batches) == 4
        o, g = both(sc, queue=bool(it & 1))       # both hand-over forms take part
        o.o.set_prev_norm(prev_o)
        g.agg.set_prev_norm(prev_g)
        ref = run_iteration(o, sc, bound)
        got = run_iteration(g, sc, bound)
        stats = compare_results(got, ref, sc)
        prev_o, prev_g = ref["norm"], got["norm"]
        nb_o = orc.policy_linear(ref["rel_delta"], pol["eta"], pol["lo_ppm"], pol["hi_ppm"])
        nb_g = dblp.policy_linear(got["rel_delta"], pol["eta"], pol["lo_ppm"], pol["hi_ppm"])
        assert nb_o == nb_g, (it, ref["rel_delta"], got["rel_delta"])
        seen.append(bound); rounds.append(ref["rounds"])
        bound = nb_o
    record_stat("cfg5_schedule_scaled_down", dict(bounds=seen, rounds=rounds, **stats))
    assert len(set(seen)) >= 3 and 20_000 in seen and max(seen) >= 140_000, seen
    assert any(20_000 < b < 140_000 for b in seen), seen
    assert seen.count(20_000) >= 3                # start, the iteration after it, the one after the x0.45 drop
    assert max(rounds) >= 1


def test_paper_burst_workload_with_epoch_controller():
    """The paper's own shape (3 workers, one accounting unit per worker, Table 1 tolerances) on a
    small gradient: 3 epochs of 3 iterations, a 70 % whole-iteration burst in a non-critical epoch.
    GPU and oracle run the retransmission loop under the epoch-level controller of Alg. Server."""
    import oracle as orc
    import paper_2605_01989_amd as dblp
    w = wl.scaled_down(wl.paper_model_workload("effnetb0", 0.7, burst_iters=(7,), iterations=9), 200_000)
    w = dataclasses.replace(w, scale_schedule=(1, 1, 1, 0.4, 0.4, 0.4, 0.4, 0.4, 0.4))
    lo, hi = w.policy["low_ppm"], w.policy["high_ppm"]
    assert (lo, hi) == (8000, 408000) and w.layout.B == 1 and w.layout.W == 3
    ctl = dblp.ClrController(lo, hi, 3)
    bound, crit, prev_o, prev_g, rounds, bounds = lo, [], None, None, [], []
    for it in range(9):
        sc = build_scenario(w, it)
        o, g = both(sc)
        o.o.set_prev_norm(prev_o)
        g.agg.set_prev_norm(prev_g)
        ref = run_iteration(o, sc, bound)
        got = run_iteration(g, sc, bound)
        compare_results(got, ref, sc)
        prev_o, prev_g = ref["norm"], got["norm"]
        rounds.append(ref["rounds"]); bounds.append(bound)
        crit.append(ref["critical"])
        bound = ctl.step(got["critical"])
        assert bound == int(orc.clr_trace(lo, hi, 3, crit)[-1])
    assert bounds == [lo, lo, lo, lo, lo, lo, lo, hi, hi]     # epoch 0 and 1 critical, epoch 2 not
    assert rounds[7] == 2          # missing after the first transmission 0.7, then 0.49, then 0.343 <= 0.408
    assert max(rounds[:7]) <= 2


# ------------------------------------------------------------------------------ sender side / broadcast leg
def test_packetize_list_rebuilds_exactly_the_listed_packets():
    """Alg. DBLP Send: only the lost packets are sent again.  The list-driven packetiser must emit
    byte-for-byte the packets the oracle's packetiser makes for the same (worker, seq) entries, and
    applying them must complete the round exactly like re-delivering the original slots."""
    import torch
    sc = build_scenario(mk(5, [366 * 120 + 9, 700, 3], 366, 0.15, place="shuffle", order="shuffle"))
    L = sc.L
    o, g = both(sc)
    for rx in (o, g):
        rx.begin_round(sc.rnd_id)
        b = sc.batches[0]
        rx.apply(b.slot_base, b.n_slots, b.mask, b.order)
    mo, lo, co, _ = o.loss_account(0)
    mg, lg, cg, _ = g.loss_account(0)
    assert np.array_equal(lo, lg) and co == cg > 0
    d_grads = [torch.from_numpy(sc.grad(w)).cuda() for w in range(L.W)]
    d_pk = torch.zeros(cg * L.stride, dtype=torch.uint8, device="cuda")
    d_src = torch.zeros(cg, dtype=torch.int16, device="cuda")
    g.agg.packetize_list(sc.rnd_id, d_grads, g.d_list, cg, d_pk, d_src)
    ref_pk = np.zeros(co * L.stride, dtype=np.uint8)
    ref_src = np.zeros(co, dtype=np.uint16)
    for i, e in enumerate(lo.tolist()):
        o.o.packetize(e >> 32, sc.rnd_id, sc.grad(e >> 32), 0, e & 0xFFFFFFFF, 1, ref_pk, ref_src, slot_base=i)
    assert np.array_equal(d_pk.cpu().numpy(), ref_pk)
    assert np.array_equal(d_src.cpu().numpy().view(np.uint16), ref_src)
    g.agg.apply_arrivals(d_pk, d_src, cg)                      # resend everything, nothing lost
    o.o.apply_arrivals(ref_pk, ref_src, co)
    assert g.loss_account(0)[3] and o.loss_account(0)[3]
    assert g.counters() == o.counters()
    full = np.ones((L.W, L.n_pkts), np.uint8)
    assert np.array_equal(g.bitmap(), full)
    from harness import abs_scale
    ref = o.finalize()
    assert np.allclose(ref, definition_mean(sc, full), rtol=1e-14, atol=0)
    assert (np.abs(g.finalize().astype(np.float64) - ref) / abs_scale(sc, full)).max() <= FLOAT_TOL
    bad = torch.tensor([(7 << 32) | 1], dtype=torch.int64, device="cuda")     # worker 7 of 5
    from paper_2605_01989_amd import DblpError
    with pytest.raises(DblpError):
        g.agg.packetize_list(sc.rnd_id, d_grads, bad, 1, d_pk, d_src)


def test_broadcast_leg_each_receiver_reconstructs_with_zero_fill():
    """Alg. Server, last statement, and Alg. Worker: the mean is sent back with DBLP_SEND; every worker
    is an independent receiver (no sum): what it lost stays zero.  One single-sender context per
    receiver; the sender's packets are built once from the aggregated gradient."""
    import torch
    import oracle as orc
    import paper_2605_01989_amd as dblp
    sc = build_scenario(mk(3, [366 * 50 + 17, 901], 366, 0.0))
    L = sc.L
    o, g = both(sc)
    ref = run_iteration(o, sc, 0)
    got = run_iteration(g, sc, 0)
    mean = g.d_out                                            # device tensor, the server's result
    bc = dblp.Aggregator(1, L.N, L.P, L.bucket_off, L.bucket_cnt)
    pk = torch.zeros(L.n_pkts * L.stride, dtype=torch.uint8, device="cuda")
    src = torch.zeros(L.n_pkts, dtype=torch.int16, device="cuda")
    bc.packetize(0, 9, mean, 0, 0, L.n_pkts, pk, src)
    oc = orc.Oracle(1, L.N, L.P, L.bucket_off, L.bucket_cnt)
    opk = np.zeros(L.n_pkts * L.stride, dtype=np.uint8)
    osrc = np.zeros(L.n_pkts, dtype=np.uint16)
    oc.packetize(0, 9, got["out"], 0, 0, L.n_pkts, opk, osrc)
    assert np.array_equal(pk.cpu().numpy(), opk)
    out = torch.empty(L.N, dtype=torch.float32, device="cuda")
    for r in range(3):                                        # three receivers, three loss patterns
        surv = wl.survive_bernoulli(sc.w.seed, 0, 10 + r, 1, L.n_pkts, 0.2)
        words = np.packbits(np.pad(surv[0], (0, (-L.n_pkts) % 64)), bitorder="little").view(np.uint64)
        bc.begin_round(9)
        bc.apply_arrivals(pk, src, L.n_pkts, torch.from_numpy(words.view(np.int64)).cuda())
        bc.finalize(out)
        oc.begin_round(9)
        oc.apply_arrivals(opk, osrc, L.n_pkts, words)
        want = oc.finalize()
        assert np.array_equal(out.cpu().numpy().astype(np.float64), want)     # one sender: exact
        pkt_of = np.concatenate([int(L.first_seq[b]) + np.arange(int(L.bucket_cnt[b])) // L.P for b in range(L.B)])
        assert np.all(want[surv[0, pkt_of] == 0] == 0.0) and np.any(want != 0)


# ------------------------------------------------------------------------------ randomized sweep
@pytest.mark.parametrize("seed", range(48))
def test_random_geometry_sweep(seed):
    """Seeded random worker counts, packet lengths, bucket tables, loss rates, placements, orders
    and bounds; two iterations each so the stored previous norm is exercised."""
    rng = np.random.default_rng(1000 + seed)
    W = int(rng.choice([1, 2, 3, 4, 5, 7, 8, 12, 16, 17, 31, 32, 33, 48, 64]))
    P = int(rng.choice([1, 2, 5, 16, 61, 62, 63, 64, 100, 254, 255, 256, 257, 366, 510, 511, 1024, 1500, 2900]))
    n_b = int(rng.integers(1, 9))
    sizes = [int(x) for x in np.maximum(1, (rng.lognormal(0, 1.5, n_b) * P * rng.integers(1, 40)).astype(np.int64))]
    while sum(sizes) * W > 6_000_000:
        sizes = [max(1, s // 2) for s in sizes]
    loss = float(rng.choice([0.0, 0.01, 0.1, 0.5, 0.95]))
    ppm = int(rng.choice([0, 8_000, 50_000, 408_000, 1_000_000]))
    place = str(rng.choice(["worker_major", "interleave", "shuffle"]))
    order = str(rng.choice(["identity", "reverse", "shuffle"]))
    w = mk(W, sizes, P, loss, seed=seed, place=place, order=order)
    # hand-over form and accumulator arrangement rotate with the seed: tables / receive queues,
    # one copy / second copy only / copies alternating per batch
    gpu_kw = [dict(), dict(acc_copies=2, acc_policy=2), dict(acc_copies=2, acc_policy=3)][seed % 3]
    prev_o = prev_g = None
    for it in range(2):
        sc = build_scenario(w, it)
        o, g = both(sc, queue=bool((seed // 3) % 2), **gpu_kw)
        o.o.set_prev_norm(prev_o)
        g.agg.set_prev_norm(prev_g)
        ref = run_iteration(o, sc, ppm)
        got = run_iteration(g, sc, ppm)
        compare_results(got, ref, sc)
        prev_o, prev_g = ref["norm"], got["norm"]


def test_early_stop_sub_batches_match_oracle():
    """Arrivals cut into sub-batches with a probe after each, stopping at the first satisfied probe:
    order-dependent, so not part of the graded path, but GPU and oracle must still agree."""
    import sys, os
    sys.path.insert(0, os.path.dirname(os.path.dirname(os.path.abspath(__file__))))
    from study_stop_granularity import run_early_stop
    from harness import abs_scale
    sc = build_scenario(mk(4, [366 * 500 + 3], 366, 0.02, place="interleave", order="shuffle"))
    o, g = both(sc)
    for k in (1, 37, 200):
        ref = run_early_stop(o, sc, 50_000, k)
        got = run_early_stop(g, sc, 50_000, k)
        assert (got["probes"], got["met"], got["accepted"]) == (ref["probes"], ref["met"], ref["accepted"])
        assert np.array_equal(got["bitmap"], ref["bitmap"])
        scale = abs_scale(sc, ref["bitmap"])
        nz = scale > 0
        assert (np.abs(got["out"] - ref["out"])[nz] / scale[nz]).max() <= FLOAT_TOL
    assert ref["probes"] < 200 and ref["accepted"] < sc.survive0.sum()      # it did stop early
