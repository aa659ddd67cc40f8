"""The entry point that allocates nothing (dblp_sumsq_static) against the one it is a variant of
(dblp_phase_signal on a vector), through the C-ABI: two calls in a row on one GPU, the second on
a smaller input, so that what the first call left in the static scratch array must not show."""
import math

import numpy as np
import pytest

import workloads as wl

pytestmark = pytest.mark.gpu


def _context(n):
    import paper_2605_01989_amd as dblp
    off, cnt = wl.buckets_from_sizes([n])
    return dblp.Aggregator(2, n, 1000, off, cnt)


def test_static_sum_of_squares_matches_phase_signal_on_two_calls_in_a_row():
    import torch
    import paper_2605_01989_amd as dblp
    from paper_2605_01989_amd import DblpError, binding
    n1, n2 = 9_000_003, 70_001          # several thousand blocks of partial sums, then a few dozen; ragged tails
    v1 = torch.from_numpy(wl.grad_values(wl.MASTER_SEED, 0, 0, 0, n1, 1e-3)).cuda()
    v2 = torch.from_numpy(wl.grad_values(wl.MASTER_SEED, 1, 0, 0, n2, 5.0)).cuda()      # larger values than the first call's
    out = torch.full((2,), -1.0, dtype=torch.float64, device="cuda")
    ref1 = _context(n1).phase_signal(v1)[0]
    ref2 = _context(n2).phase_signal(v2)[0]
    torch.cuda.synchronize()
    free_before = torch.cuda.mem_get_info()[0]
    dblp.sumsq_static(v1, out[0:1])
    dblp.sumsq_static(v2, out[1:2])
    torch.cuda.synchronize()
    assert torch.cuda.mem_get_info()[0] == free_before           # no device memory was taken
    got = out.cpu().numpy()
    assert math.sqrt(got[0]) == ref1 and math.sqrt(got[1]) == ref2      # same arithmetic, same block order: same bits
    for v, g in ((v1, got[0]), (v2, got[1])):
        want = float((v.cpu().numpy().astype(np.float64) ** 2).sum())
        assert abs(g - want) <= 1e-9 * want
    # the smaller call again, after the larger one once more: still the same bits
    dblp.sumsq_static(v1, out[0:1])
    dblp.sumsq_static(v2, out[1:2])
    torch.cuda.synchronize()
    assert np.array_equal(out.cpu().numpy(), got)
    # limits and arguments
    for bad in (dict(n_elems=0), dict(n_elems=(1 << 36) + 1), dict(device=16, stream=0)):
        with pytest.raises(DblpError) as e:
            dblp.sumsq_static(v2, out[1:2], **bad)
        assert e.value.code == binding.EINVAL and "sumsq_static" in str(e.value)
    with pytest.raises(DblpError) as e:
        dblp.sumsq_static(v2[1:], out[1:2])                       # not 16-byte aligned
    assert e.value.code == binding.EINVAL
