"""Pins for the CPU oracle: what the paper and plain mathematics fix, checked without
re-using the oracle's own formulas.  A wrong sign, index, divisor, threshold direction or
byte order anywhere in oracle/dblp_oracle.c fails at least one of these."""
import itertools
import math
import os

import numpy as np
import pytest

import oracle
import workloads as wl
from harness import OracleRx, build_scenario, definition_mean, run_iteration

GOLDEN = os.path.join(os.path.dirname(__file__), "golden", "paper_constants.txt")


def paper_constants():
    out = {}
    for line in open(GOLDEN):
        line = line.split("#")[0].split()
        if len(line) == 2:
            out[line[0]] = float(line[1])
    return out


def tiny(W, sizes, P, loss=0.0, seed=7, place="worker_major", order="identity"):
    off, cnt = wl.buckets_from_sizes(sizes)
    w = wl.Workload("tiny", wl.Layout(W, int(sum(sizes)), P, off, cnt), 1e-3,
                    dict(kind="bernoulli", p=loss) if loss else dict(kind="none"),
                    place, order, dict(kind="fixed", ppm=0), seed=seed)
    return w


def fresh(sc):
    rx = OracleRx(sc)
    rx.packetize_all()
    rx.begin_round(sc.rnd_id)
    return rx


# ---------------------------------------------------------------- wire format
def test_header_is_little_endian_seq_round_len_and_mtu_sized():
    """Sec. Metadata: three header fields.  366 floats + 8-byte header = 1472 bytes, the UDP
    payload of a 1500-byte MTU (1500 - 20 IP - 8 UDP)."""
    sc = build_scenario(tiny(1, [366 * 300 + 5], 366))
    assert sc.L.stride == 1472 == 1500 - 20 - 8
    rx = OracleRx(sc)
    rx.packetize_all(rnd_id=0xBEEF)
    p = rx.packets.reshape(-1, 1472)
    assert bytes(p[258, :8]) == bytes([0x02, 0x01, 0, 0, 0xEF, 0xBE, 0x6E, 0x01])  # seq 258, len 366
    assert bytes(p[300, :8]) == bytes([0x2C, 0x01, 0, 0, 0xEF, 0xBE, 5, 0])        # short tail packet
    g = sc.grad(0)
    assert np.array_equal(p[258, 8:8 + 1464].view(np.float32), g[258 * 366:259 * 366])
    assert np.array_equal(p[300, 8:8 + 20].view(np.float32), g[300 * 366:])
    assert not p[300, 28:].any()


def test_packets_do_not_straddle_buckets():
    sc = build_scenario(tiny(1, [5, 3, 4], 2))
    rx = OracleRx(sc)
    rx.packetize_all()
    p = rx.packets.reshape(-1, sc.L.stride)
    lens = p[:, 6].astype(int) | p[:, 7].astype(int) << 8
    assert lens.tolist() == [2, 2, 1, 2, 1, 2, 2]


# ---------------------------------------------------------------- brute force
@pytest.mark.parametrize("W,sizes,P", [(2, [3], 2), (3, [2, 1], 1), (1, [5], 2)])
def test_brute_force_all_masks_all_permutations(W, sizes, P):
    """Every loss mask and every arrival order on a tiny gradient against the one-line
    definition out[e] = (1/W) sum_w m[w, pkt(e)] g[w, e]."""
    sc = build_scenario(tiny(W, sizes, P))
    L = sc.L
    n = L.W * L.n_pkts
    rx = OracleRx(sc)
    rx.packetize_all()
    for maskbits in range(1 << n):
        m = np.array([(maskbits >> s) & 1 for s in range(n)], dtype=np.uint8).reshape(L.W, L.n_pkts)
        want = definition_mean(sc, m)
        words = wl.slot_mask_words(m, sc.slot_of)
        for perm in itertools.permutations(range(n)):
            rx.begin_round(sc.rnd_id)
            rx.apply(0, n, words, np.array(perm, dtype=np.uint32))
            got = rx.finalize()
            assert np.allclose(got, want, rtol=1e-15, atol=0), (maskbits, perm)
            assert np.array_equal(rx.bitmap(), m)
            if n > 4:
                break  # all permutations only on the smallest cases; others: first one per mask


def test_brute_force_random_masks_random_permutations_ragged():
    sc = build_scenario(tiny(3, [7, 1, 12, 4], 3, seed=11))
    L = sc.L
    n = L.W * L.n_pkts
    rx = OracleRx(sc)
    rx.packetize_all()
    rng = np.random.default_rng(5)
    for _ in range(200):
        m = (rng.random((L.W, L.n_pkts)) < 0.6).astype(np.uint8)
        rx.begin_round(sc.rnd_id)
        rx.apply(0, n, wl.slot_mask_words(m, sc.slot_of), rng.permutation(n).astype(np.uint32))
        assert np.allclose(rx.finalize(), definition_mean(sc, m), rtol=1e-15, atol=0)
        assert np.array_equal(rx.bitmap(), m)


# ---------------------------------------------------------------- closed forms
def test_zero_loss_is_the_exact_mean():
    """Alg. Server: mean over all workers.  Summed in worker order, bit-for-bit numpy's mean."""
    sc = build_scenario(tiny(4, [1000, 37, 2048], 16, place="worker_major"))
    rx = fresh(sc)
    rx.apply(0, sc.L.W * sc.L.n_pkts, None, None)
    stack = np.stack([sc.grad(w).astype(np.float64) for w in range(4)])
    want = ((stack[0] + stack[1]) + stack[2] + stack[3]) / 4
    assert np.array_equal(rx.finalize(), want)
    assert np.allclose(rx.finalize(), stack.mean(axis=0), rtol=1e-15)
    assert rx.counters() == dict(accepted=4 * sc.L.n_pkts, duplicate=0, stale=0, invalid=0)


def test_one_worker_entirely_lost_divides_by_all_workers():
    """Zero-fill then mean over ALL workers: losing worker 2 gives (sum of the others)/W,
    not the mean of the survivors."""
    sc = build_scenario(tiny(3, [500], 8))
    rx = fresh(sc)
    m = np.ones((3, sc.L.n_pkts), dtype=np.uint8)
    m[2] = 0
    rx.apply(0, 3 * sc.L.n_pkts, wl.slot_mask_words(m, sc.slot_of), None)
    want = (sc.grad(0).astype(np.float64) + sc.grad(1).astype(np.float64)) / 3
    assert np.allclose(rx.finalize(), want, rtol=1e-15)
    missing, lst, count, met = rx.loss_account(1_000_000)     # 100 % tolerance: nothing to resend
    assert met and count == 0 and missing[2, 0] == sc.L.n_pkts


def test_never_received_elements_are_exactly_zero():
    sc = build_scenario(tiny(2, [64], 4))
    rx = fresh(sc)
    m = np.ones((2, 16), dtype=np.uint8)
    m[:, 5] = 0
    rx.apply(0, 32, wl.slot_mask_words(m, sc.slot_of), None)
    out = rx.finalize()
    assert np.all(out[20:24] == 0.0) and np.all(out[:20] != 0.0)


def test_second_moment_matches_zero_fill_over_W_convention():
    """i.i.d. N(0, s^2) inputs, i.i.d. loss q: E||out||^2 = N s^2 (1-q) / W.  Dividing by the
    received count instead of W would give a different constant."""
    W, N, q, s = 4, 400_000, 0.25, 1e-3
    sc = build_scenario(tiny(W, [N], 100, loss=q))
    rx = fresh(sc)
    b = sc.batches[0]
    rx.apply(0, b.n_slots, b.mask, None)
    out = rx.finalize()
    want = N * s * s * (1 - q) / W
    assert abs(float(out @ out) / want - 1) < 0.02


def test_linearity_masking_inputs_equals_masking_packets():
    sc = build_scenario(tiny(2, [300, 45], 7, loss=0.3))
    rx = fresh(sc)
    b = sc.batches[0]
    rx.apply(0, b.n_slots, b.mask, None)
    assert np.allclose(rx.finalize(), definition_mean(sc, sc.survive0), rtol=1e-15)


# ---------------------------------------------------------------- order / duplicates / stale
def test_permutation_invariance():
    """Property 1 of the paper: no reliance on in-order delivery."""
    sc = build_scenario(tiny(4, [4000, 333], 16, loss=0.1, order="shuffle"))
    ref = run_iteration(fresh(sc), sc, 50_000)
    for order in ("identity", "reverse"):
        sc2 = build_scenario(tiny(4, [4000, 333], 16, loss=0.1, order=order))
        got = run_iteration(fresh(sc2), sc2, 50_000)
        assert np.array_equal(got["bitmap"], ref["bitmap"])
        assert [p["count"] for p in got["probes"]] == [p["count"] for p in ref["probes"]]
        assert all(np.array_equal(a["list"], b["list"]) for a, b in zip(got["probes"], ref["probes"]))
        assert np.allclose(got["out"], ref["out"], rtol=1e-14, atol=0)


def test_stale_round_packets_are_dropped_and_counted():
    """A packet of round k arriving during round k+1 is dropped."""
    sc = build_scenario(tiny(2, [100], 10))
    rx = OracleRx(sc)
    rx.packetize_all(rnd_id=sc.rnd_id - 1)
    rx.begin_round(sc.rnd_id)
    rx.apply(0, 20, None, None)
    assert rx.counters() == dict(accepted=0, duplicate=0, stale=20, invalid=0)
    assert not rx.finalize().any() and not rx.bitmap().any()


def test_duplicates_are_ignored_first_copy_wins():
    sc = build_scenario(tiny(2, [100], 10))
    rx = fresh(sc)
    order = np.concatenate([np.arange(20), np.arange(20), [3, 3]]).astype(np.uint32)
    rx.apply(0, 20, None, order)
    assert rx.counters() == dict(accepted=20, duplicate=22, stale=0, invalid=0)
    assert np.allclose(rx.finalize(), definition_mean(sc, np.ones((2, 10), np.uint8)), rtol=1e-15)
    rx.apply(0, 20, None, None)   # a whole second batch of the same packets
    assert rx.counters()["duplicate"] == 42
    assert np.allclose(rx.finalize(), definition_mean(sc, np.ones((2, 10), np.uint8)), rtol=1e-15)


def test_invalid_packets_are_rejected():
    sc = build_scenario(tiny(2, [100, 7], 10))   # 11 packets per worker, last one 7 floats
    rx = fresh(sc)
    p = rx.packets.reshape(-1, sc.L.stride)
    p[0, 0:4] = np.frombuffer(np.uint32(11).tobytes(), np.uint8)        # seq out of range
    p[1, 6:8] = np.frombuffer(np.uint16(9).tobytes(), np.uint8)         # wrong length
    p[10, 6:8] = np.frombuffer(np.uint16(10).tobytes(), np.uint8)       # tail packet claiming full length
    rx.src[2] = 2                                                       # worker out of range
    order = np.concatenate([np.arange(22), [22, 1000]]).astype(np.uint32)   # slots out of range
    rx.apply(0, 22, None, order)
    assert rx.counters() == dict(accepted=18, duplicate=0, stale=0, invalid=6)
    m = np.ones((2, 11), np.uint8)
    m[0, [0, 1, 2, 10]] = 0
    assert np.array_equal(rx.bitmap(), m)
    assert np.allclose(rx.finalize(), definition_mean(sc, m), rtol=1e-15)


@pytest.mark.parametrize("threads", [1, 3, 8])
def test_thread_parallel_walk_equals_the_plain_walk_bit_for_bit(threads):
    """The all-cores baseline splits the reconstruction buffer into disjoint element ranges, one per
    thread; nothing observable may differ from the single-threaded arrival-order walk: bitmap,
    the four counters, the fp64 sums (bitwise), lists and counts, with duplicates whose payloads
    conflict, stale, invalid and lost packets in the stream."""
    sc = build_scenario(tiny(5, [366 * 37 + 9, 1, 700, 366 * 4, 50], 366, loss=0.1, seed=17, place="shuffle", order="shuffle"))
    L = sc.L
    n = L.W * L.n_pkts
    a, b = fresh(sc), fresh(sc)
    for rx in (a, b):
        p = rx.packets.reshape(-1, L.stride)
        p[5, 4:6] = np.frombuffer(np.uint16(sc.rnd_id + 1).tobytes(), np.uint8)     # stale
        p[6, 4:6] = np.frombuffer(np.uint16(sc.rnd_id + 1).tobytes(), np.uint8)     # stale and ...
        p[6, 0:4] = np.frombuffer(np.uint32(L.n_pkts + 9).tobytes(), np.uint8)      # ... seq out of range
        p[9, 6:8] = np.frombuffer(np.uint16(3).tobytes(), np.uint8)                  # wrong length
        p[11, 0:4] = np.frombuffer(np.uint32(L.n_pkts).tobytes(), np.uint8)          # seq out of range
        rx.src[20] = L.W                                                             # worker out of range
        p[30, 0:8] = p[31, 0:8]                      # slot 30 now claims to be slot 31's packet,
        rx.src[30] = rx.src[31]                      # from the same worker: a copy with a conflicting payload
    bt = sc.batches[0]
    order = np.concatenate([bt.order, bt.order[:60], [n + 3]]).astype(np.uint32)
    a.apply(0, n, bt.mask, order)
    used = b.o.apply_arrivals(b.packets, b.src, n, bt.mask, order, threads=threads)
    assert used == threads
    for rnd in range(1, 3):
        ma, la, ca, meta = a.loss_account(30_000)
        mb, lb, cb, metb = b.loss_account(30_000)
        assert np.array_equal(ma, mb) and np.array_equal(la, lb) and (ca, meta) == (cb, metb)
        slots = sc.resend(la, rnd)
        a.apply(0, n, None, slots)
        b.o.apply_arrivals(b.packets, b.src, n, None, slots, threads=threads)
    assert a.counters() == b.counters() and a.counters()["duplicate"] >= 50 and a.counters()["invalid"] >= 4
    assert np.array_equal(a.bitmap(), b.bitmap())
    assert np.array_equal(a.o.acc().view(np.uint64), b.o.acc().view(np.uint64))


def test_header_writer_gives_the_first_eight_bytes_of_every_packet():
    """The header-only sender must write exactly what the packetiser puts in front of the payload,
    at the same slots (ragged buckets, shuffled placement)."""
    sc = build_scenario(tiny(3, [366 * 41 + 9, 1, 700, 366 * 3], 366, seed=13, place="shuffle"))
    L = sc.L
    n = L.W * L.n_pkts
    rx = OracleRx(sc)
    rx.packetize_all(rnd_id=0xA1B2)
    headers = np.full(n * 8, 0xEE, dtype=np.uint8)
    src = np.full(n, 0xFFFF, dtype=np.uint16)
    for w in range(L.W):
        rx.o.write_headers(w, 0xA1B2, 0, L.n_pkts, headers, src, slot_map=sc.slot_of[w])
    assert np.array_equal(headers.reshape(n, 8), rx.packets.reshape(n, L.stride)[:, :8])
    assert np.array_equal(src, rx.src)
    lens = headers.reshape(n, 8)[:, 6].astype(int) | headers.reshape(n, 8)[:, 7].astype(int) << 8
    assert sorted(set(lens.tolist())) == [1, 9, 334, 366]        # 700 = 366 + 334: short tails carry their own length


def test_header_only_mode_gives_the_integer_outputs_of_the_full_receiver():
    """Alg. DBLP_RECV decides acceptance from the header alone (round, sequence number, length):
    a receiver that is shown only the 8 header bytes of every slot must end with the bitmap,
    counters, per-bucket counts and retransmit lists of one that also adds the payloads, through
    retransmission rounds, with stale, invalid, duplicate and lost packets in the stream."""
    sc = build_scenario(tiny(3, [366 * 41 + 9, 1, 700, 366 * 3], 366, loss=0.15, seed=13, place="shuffle", order="shuffle"))
    L = sc.L
    n = L.W * L.n_pkts
    full = fresh(sc)
    p = full.packets.reshape(-1, L.stride)
    p[5, 4:6] = np.frombuffer(np.uint16(sc.rnd_id + 1).tobytes(), np.uint8)     # stale
    p[9, 6:8] = np.frombuffer(np.uint16(3).tobytes(), np.uint8)                  # wrong length
    p[11, 0:4] = np.frombuffer(np.uint32(L.n_pkts).tobytes(), np.uint8)          # seq out of range
    full.src[20] = L.W                                                           # worker out of range
    headers = np.ascontiguousarray(p[:, :8]).reshape(-1)                         # nothing but the headers
    lean = oracle.Oracle(L.W, L.N, L.P, L.bucket_off, L.bucket_cnt)
    lean.begin_round(sc.rnd_id)
    b = sc.batches[0]
    order = np.concatenate([b.order, b.order[:50], [n + 3]]).astype(np.uint32)   # duplicates, a slot outside
    full.apply(0, n, b.mask, order)
    lean.apply_arrivals(headers, full.src, n, b.mask, order, accumulate=False, stride=8)
    for rounds in range(1, 5):      # the corrupted packets are never accepted, so the loop is cut, not run until met
        m0, l0, c0, met0 = full.loss_account(20_000)
        m1, l1, c1, met1 = lean.loss_account(20_000)
        assert np.array_equal(m0, m1) and np.array_equal(l0, l1) and (c0, met0) == (c1, met1) and not met0
        assert np.array_equal(full.bitmap(), lean.received()) and full.counters() == lean.counters()
        slots = sc.resend(l0, rounds)
        full.apply(0, n, None, slots)
        lean.apply_arrivals(headers, full.src, n, None, slots, accumulate=False, stride=8)
    assert np.array_equal(full.bitmap(), lean.received()) and full.counters() == lean.counters()
    assert full.counters()["duplicate"] >= 40 and full.counters()["stale"] >= 1
    assert full.counters()["invalid"] >= 3
    assert not lean.acc().any() and full.o.acc().any()          # payloads were never touched


# ---------------------------------------------------------------- tolerance test
@pytest.mark.parametrize("n_b,ppm,allowed", [(64, 50_000, 3), (125, 8_000, 1), (1, 150_000, 0),
                                             (366, 24_000, 8), (250, 8_000, 2), (1000, 408_000, 408)])
def test_threshold_is_inclusive_and_rounds_down(n_b, ppm, allowed):
    """'equal to or less than the loss value p': missing/n <= p.  Hand-computed allowed counts:
    0.05*64=3.2 -> 3; 0.008*125=1 -> 1 (boundary passes); 0.15*1 -> 0; 0.024*366=8.78 -> 8;
    0.008*250=2 -> 2 (boundary passes); 0.408*1000=408."""
    sc = build_scenario(tiny(1, [n_b * 2], 2))
    for miss, ok in ((allowed, True), (allowed + 1, False)):
        if miss > n_b:
            continue
        rx = fresh(sc)
        m = np.ones((1, n_b), np.uint8)
        m[0, :miss] = 0
        rx.apply(0, n_b, wl.slot_mask_words(m, sc.slot_of), None)
        missing, lst, count, met = rx.loss_account(ppm)
        assert missing[0, 0] == miss and met == ok
        assert count == (0 if ok else miss)
        if not ok:
            assert lst.tolist() == list(range(miss))


def test_retransmit_list_only_failing_buckets_sorted_and_sufficient():
    sc = build_scenario(tiny(3, [640, 640, 640, 100], 10, loss=0.08, seed=3))
    rx = fresh(sc)
    b = sc.batches[0]
    rx.apply(0, b.n_slots, b.mask, None)
    missing, lst, count, met = rx.loss_account(80_000)     # allowed: 5,5,5,0 of 64,64,64,10
    L = sc.L
    allowed = (80_000 * L.n_b.astype(np.int64)) // 1_000_000
    assert allowed.tolist() == [5, 5, 5, 0]
    rec = rx.bitmap()
    # independent recount from the survival bits
    want_missing = np.array([[int((1 - sc.survive0[w, int(L.first_seq[bb]):int(L.first_seq[bb + 1])]).sum())
                              for bb in range(L.B)] for w in range(L.W)])
    assert np.array_equal(missing, want_missing)
    want = [(w << 32) | s for w in range(L.W) for bb in range(L.B) if want_missing[w, bb] > allowed[bb]
            for s in range(int(L.first_seq[bb]), int(L.first_seq[bb + 1])) if not rec[w, s]]
    assert lst.tolist() == want and count == len(want) and not met and count > 0
    assert lst.tolist() == sorted(lst.tolist())
    # resending the whole list without loss satisfies every bucket
    slots = sc.slot_of[(lst >> np.uint64(32)).astype(int), (lst & np.uint64(0xFFFFFFFF)).astype(int)]
    rx.apply(0, b.n_slots, None, slots.astype(np.uint32))
    missing2, lst2, count2, met2 = rx.loss_account(80_000)
    assert met2 and count2 == 0 and np.all(missing2 <= allowed[None, :])
    # identity: total missing = packets - accepted
    assert int(missing2.sum()) == L.W * L.n_pkts - rx.counters()["accepted"]


def test_list_capacity_truncates_but_reports_full_count():
    sc = build_scenario(tiny(1, [40], 2))
    rx = fresh(sc)
    missing, lst, count, met = rx.o.loss_account(0, capacity=7)
    assert count == 20 and lst.tolist() == list(range(7)) and not met


def test_received_fraction_after_loop_meets_paper_invariant():
    """With tolerance 0.8 % the receiver ends every iteration with >= 99.2 % of the packets of
    every accounting unit (Sec. "Evaluation Accuracy Results")."""
    c = paper_constants()
    ppm = int(round(c["p_low_effnetb0_percent"] * 10_000))
    assert ppm == 8000 and 100 - c["p_low_effnetb0_percent"] == c["processed_at_0p8_percent"]
    sc = build_scenario(tiny(3, [125 * 20] * 4 + [1000 * 20], 20, loss=0.05, seed=9, order="shuffle"))
    res = run_iteration(fresh(sc), sc, ppm)
    L = sc.L
    assert res["rounds"] >= 1
    for w in range(L.W):
        for b in range(L.B):
            got = res["bitmap"][w, int(L.first_seq[b]):int(L.first_seq[b + 1])].mean()
            assert got >= c["processed_at_0p8_percent"] / 100 - 1e-12
    assert np.allclose(res["out"], definition_mean(sc, res["bitmap"]), rtol=1e-14)


def test_single_bucket_reproduces_whole_round_accounting():
    """One bucket over the whole gradient = the paper's ratio over all chunks of a cycle."""
    sc = build_scenario(tiny(2, [3000], 3, loss=0.1, seed=21))
    rx = fresh(sc)
    b = sc.batches[0]
    rx.apply(0, b.n_slots, b.mask, None)
    lost = (1 - sc.survive0).sum(axis=1)
    for ppm in (50_000, 100_000, 150_000):
        missing, lst, count, met = rx.loss_account(ppm)
        fails = [w for w in range(2) if lost[w] / 1000 > ppm / 1e6]
        assert count == sum(int(lost[w]) for w in fails) and met == (not fails)


# ---------------------------------------------------------------- phase signal (Eq. 1)
def test_phase_signal_truth_table_and_norm():
    c = paper_constants()
    o = oracle.Oracle(1, 16, 4, [0], [16], eta=c["eta"])
    v = np.full(16, 3.0)
    norm, delta, crit = o.phase_signal(v)
    assert norm == 12.0 == 3.0 * math.sqrt(16) and crit and math.isinf(delta)   # first iteration is critical
    for prev, cur, want in [(1.0, 0.5, True), (1.0, 1.5, True), (1.0, 0.51, False), (1.0, 1.0, False),
                            (2.0, 0.99, True), (2.0, 3.01, True), (2.0, 2.9, False)]:
        o.set_prev_norm(prev)
        norm, delta, crit = o.phase_signal(np.full(16, cur / 4.0))
        assert norm == pytest.approx(cur, rel=1e-15)
        assert delta == pytest.approx(abs(prev - cur) / prev, rel=1e-12) and crit == want
    # previous norm is replaced by the current one
    o.set_prev_norm(1.0)
    o.phase_signal(np.full(16, 2.0))
    _, delta, _ = o.phase_signal(np.full(16, 1.0))
    assert delta == pytest.approx(0.5)
    o.set_prev_norm(0.0)
    assert o.phase_signal(v)[2] is True


def test_two_level_policy_matches_table_1():
    c = paper_constants()
    for m in ("effnetb0", "resnet50", "alexnet", "gpt2s"):
        lo = int(round(c[f"p_low_{m}_percent"] * 10_000))
        hi = int(round(c[f"p_high_{m}_percent"] * 10_000))
        assert hi - lo == int(c["k_percent"]) * 10_000
        assert oracle.policy_two_level(True, lo, hi) == lo
        assert oracle.policy_two_level(False, lo, hi) == hi


def test_extension_policies_follow_their_definitions():
    """Not paper content (parity unpinned by the paper): three levels at eta and eta/2; linear ramp."""
    assert oracle.policy_three_level(0.5, 0.5, 10_000, 50_000, 100_000) == 10_000
    assert oracle.policy_three_level(0.49, 0.5, 10_000, 50_000, 100_000) == 50_000
    assert oracle.policy_three_level(0.25, 0.5, 10_000, 50_000, 100_000) == 50_000
    assert oracle.policy_three_level(0.2499, 0.5, 10_000, 50_000, 100_000) == 100_000
    assert oracle.policy_three_level(math.inf, 0.5, 10_000, 50_000, 100_000) == 10_000
    assert oracle.policy_linear(0.0, 0.5, 20_000, 150_000) == 150_000
    assert oracle.policy_linear(0.5, 0.5, 20_000, 150_000) == 20_000
    assert oracle.policy_linear(math.inf, 0.5, 20_000, 150_000) == 20_000
    assert oracle.policy_linear(0.25, 0.5, 20_000, 150_000) == 85_000
    assert oracle.policy_linear(0.1, 0.5, 20_000, 150_000) == 124_000


def test_create_rejects_bad_tables():
    with pytest.raises(ValueError):
        oracle.Oracle(2, 10, 4, [0, 6], [5, 4])      # gap
    with pytest.raises(ValueError):
        oracle.Oracle(2, 10, 4, [0, 5], [5, 4])      # does not reach N
    with pytest.raises(ValueError):
        oracle.Oracle(0, 10, 4, [0], [10])


def test_epoch_controller_follows_the_server_algorithm():
    """Alg. Server: threshold starts at P_low; only the first step of an epoch re-decides: reset to
    P_high, back to P_low if that step is critical.  Hand-traced sequence, 3 steps per epoch."""
    lo, hi = 8000, 408000
    crit = [1, 0, 0,   0, 1, 1,   1, 0, 0,   0, 0, 0]
    want = [lo, lo, lo, hi, hi, hi, lo, lo, lo, hi, hi, hi]
    assert oracle.clr_trace(lo, hi, 3, crit).tolist() == want
    # one step per epoch degenerates to the per-iteration two-level rule
    assert oracle.clr_trace(lo, hi, 1, [1, 0, 1, 0]).tolist() == [lo, hi, lo, hi]


# ------------------------------------------------------------------------------ receive-queue form
def test_receive_queue_is_the_same_batch_to_the_oracle():
    """The test harness turns (per-slot worker table, mask, order) into receive-queue descriptors
    for the library's queue entry point.  The conversion is checked here on the CPU: feeding the
    oracle the descriptors' slots as the order and the descriptors' workers as the worker table,
    with no mask, must classify every arrival and produce every output exactly as the original
    batch does -- duplicates, stale, out-of-range slots and foreign workers included."""
    from harness import receive_queue
    off, cnt = wl.buckets_from_sizes([40 * 7 + 3, 5, 64])
    w = wl.Workload("q", wl.Layout(3, int(sum([40 * 7 + 3, 5, 64])), 7, off, cnt), 1e-3, dict(kind="bernoulli", p=0.2),
                    "shuffle", "shuffle", dict(kind="fixed", ppm=0), seed=5)
    sc = build_scenario(w)
    L = sc.L
    n = L.W * L.n_pkts
    a = OracleRx(sc); a.packetize_all()
    p = a.packets.reshape(-1, L.stride)
    p[4, 4:6] = np.frombuffer(np.uint16(sc.rnd_id + 1).tobytes(), np.uint8)      # a stale packet
    a.src[7] = 9                                                                 # a foreign worker
    rng = np.random.default_rng(1)
    order = np.concatenate([rng.permutation(n), rng.integers(0, n, 30), [n, n + 5]]).astype(np.uint32)   # duplicates, bad slots
    mask = sc.batches[0].mask
    a.begin_round(sc.rnd_id)
    a.apply(0, n, mask, order)
    q = receive_queue(a.src, n, mask, order, order.size)
    assert q.size < order.size and np.all(q >> np.uint64(48) == 0)
    b = OracleRx(sc); b.packets = a.packets
    b.src = np.zeros(n, dtype=np.uint16)
    slots = (q & np.uint64(0xFFFFFFFF)).astype(np.uint32)
    inside = slots < n
    # every slot has one worker in the table, so the queue's worker field is a function of the slot
    b.src[slots[inside]] = (q[inside] >> np.uint64(32)).astype(np.uint16)
    assert np.array_equal(b.src[np.unique(slots[inside])], a.src[np.unique(slots[inside])])
    b.begin_round(sc.rnd_id)
    b.apply(0, n, None, slots)
    assert a.counters() == b.counters() and a.counters()["stale"] >= 1 and a.counters()["invalid"] >= 3
    assert a.counters()["duplicate"] >= 1
    assert np.array_equal(a.bitmap(), b.bitmap())
    assert np.array_equal(a.finalize(), b.finalize())
    ma, la, ca, _ = a.loss_account(0)
    mb, lb, cb, _ = b.loss_account(0)
    assert np.array_equal(ma, mb) and np.array_equal(la, lb) and ca == cb
