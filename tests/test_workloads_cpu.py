"""The seeded input generators: C vs numpy restatement, geometry of the named workloads."""
import numpy as np
import pytest

import workloads as wl


def test_c_generator_matches_numpy_restatement():
    for (w, it, e0, n, tail) in [(0, 0, 0, 4097, 0), (3, 7, 123456789, 1000, 0), (31, 19, 2**33 + 5, 513, 10000)]:
        a = wl.grad_values(wl.MASTER_SEED, w, it, e0, n, 1e-3, tail, 100.0)
        b = wl.grad_values_numpy(wl.MASTER_SEED, w, it, e0, n, 1e-3, tail, 100.0)
        assert np.array_equal(a.view(np.uint32), b.view(np.uint32))


def test_values_are_roughly_normal_with_requested_std():
    x = wl.grad_values(1, 0, 0, 0, 2_000_000, 1e-3)
    assert abs(x.std() / 1e-3 - 1) < 5e-3 and abs(x.mean()) < 5e-6
    k = ((x / x.std()) ** 4).mean()
    assert 2.8 < k < 3.0          # Irwin-Hall(12): kurtosis 2.9
    assert np.unique(x).size > 100_000   # full-mantissa values, so fp32 sums do round


@pytest.mark.parametrize("name,W,N,P,B,n_pkts,stride", [
    ("cfg1", 4, 1 << 20, 256, 64, 4096, 1040),
    ("cfg2", 8, 25_600_000, 366, 161, None, 1472),
    ("cfg3", 8, 124_439_808, 366, 148, None, 1472),
    ("cfg4", 16, 354_823_168, 1024, 292, None, 4112),
    ("cfg5", 32, 1_300_000_000, 366, 868, 3_551_913, 1472)])
def test_named_workload_geometry(name, W, N, P, B, n_pkts, stride):
    L = wl.workload(name).layout
    assert (L.W, L.N, L.P, L.B, L.stride) == (W, N, P, B, stride)
    assert int(L.bucket_cnt.sum()) == N and int(L.bucket_off[0]) == 0
    assert np.array_equal(L.bucket_off[1:], np.cumsum(L.bucket_cnt)[:-1])
    if n_pkts:
        assert L.n_pkts == n_pkts


def test_loss_processes_have_the_stated_rates():
    s = wl.survive_bernoulli(5, 0, 0, 2, 500_000, 0.02)
    assert abs((1 - s.mean()) / 0.02 - 1) < 0.03
    g = wl.survive_gilbert_elliott(5, 0, 0, 4, 2_000_000, 0.001, 0.30, 1 / 1960, 1 / 40)
    assert abs((1 - g.mean()) / 0.00698 - 1) < 0.1      # 0.98*0.001 + 0.02*0.30
    # bursts: the mean run of consecutive losses is far longer than for i.i.d. loss at that rate
    lost = (g[0] == 0).astype(np.int8)
    runs = np.diff(np.flatnonzero(np.diff(np.concatenate([[0], lost, [0]]))))[::2]
    assert runs.mean() > 1.2
    slot_of = wl.placement("interleave", 4, 100_000, 9)
    m = wl.survive_microburst(5, 0, 0, slot_of, 3, 0.005, 0.005)
    assert abs((1 - m.mean()) / 0.0199 - 1) < 0.05      # 3 x 0.5 % windows + 0.5 % elsewhere


def test_placements_are_permutations_and_interleave_keeps_seq_order():
    for kind in ("worker_major", "interleave", "shuffle"):
        s = wl.placement(kind, 5, 1000, 3)
        assert sorted(s.reshape(-1).tolist()) == list(range(5000))
    s = wl.placement("interleave", 5, 1000, 3)
    assert np.all(np.diff(s.astype(np.int64), axis=1) > 0)
    L = wl.workload("cfg1").layout
    pc = wl.placement_chunked("shuffle", L, 16, 3)
    for (s0, s1) in wl.chunk_seq_ranges(L, 16):
        blk = np.sort(pc[:, s0:s1].reshape(-1))
        assert blk[0] == L.W * s0 and blk[-1] == L.W * s1 - 1 and np.all(np.diff(blk) == 1)


def test_mask_words_follow_slots():
    slot_of = wl.placement("shuffle", 2, 70, 1)
    surv = (np.arange(140).reshape(2, 70) % 3 != 0).astype(np.uint8)
    words = wl.slot_mask_words(surv, slot_of)
    for w in range(2):
        for s in range(70):
            slot = int(slot_of[w, s])
            assert (int(words[slot >> 6]) >> (slot & 63)) & 1 == surv[w, s]
