"""replay_sample_gather_static, the entry point for callers that cannot allocate: its scratch
(the slot numbers of a batch without duplicates, between the draw kernel and the gather kernel)
is a fixed array inside the library.  Through the C ABI its outputs must equal those of
replay_sample_gather bit for bit, on two calls in a row, the second with a smaller batch (the
array then still holds the first call's slot numbers beyond the new batch), and the slot numbers
must be the oracle's."""
import numpy as np
import pytest
import torch

import oracle
from paper_1801_03138_amd import synth

pytestmark = pytest.mark.gpu


@pytest.fixture(scope="module")
def B():
    from paper_1801_03138_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.lib()
    return binding


def _dev(rows, chain):
    d = {k: torch.from_numpy(v).cuda() for k, v in rows.items()}
    if chain:
        d["s_next"] = None
    return d


def _same(a, b, what):
    torch.cuda.synchronize()
    for x, y, name in zip(a, b, synth.FIELDS + ("idx",)):
        assert torch.equal(x.view(torch.uint8), y.view(torch.uint8)), (what, name)


@pytest.mark.parametrize("chain", [False, True])
def test_static_scratch_entry_point_matches_the_allocating_one(B, chain):
    C, D, seed = 100_000, 27, 17
    layout = B.RP_CHAIN if chain else B.RP_PAIR
    gpu = B.Replay(C, D, B.RP_F32, layout, seed=seed, max_append=4096, distinct=True)
    rows = synth.experiences(50_000, D, 30, 0.01, seed=3)
    d = _dev(rows, chain)
    for _ in range(3):                                   # 150,000 experiences: the ring wraps
        gpu.append(d["s"], d["s_next"], d["a"], d["r"], d["term"])
    head, size, total = gpu.state()
    choices = size - 1 if chain else size
    oldest = (head + C - size) % C
    for call, (step, batch) in enumerate([(5, 65_536), (6, 1000), (7, 3), (8, 9000)]):
        want = gpu.sample_gather(step, batch)[1]
        torch.cuda.synchronize()
        out = gpu.alloc_batch(batch)
        for t in out:
            t.view(torch.uint8).fill_(0xA5)
        st, got = gpu.sample_gather_static(step, batch, out)
        assert st == 0
        _same(got, want, "call %d" % call)
        idx = got[5].cpu().numpy().view(np.uint32)
        assert len(np.unique(idx)) == batch
        for i in sorted(set(list(range(0, batch, 499)) + [batch - 1])):
            u = oracle.distinct_index(seed, step, i, choices)
            assert idx[i] == ((oldest + u) % C if chain else u)


def test_static_scratch_entry_point_limits_and_plain_sampling(B):
    D = 27
    rows = synth.experiences(70_000, D, 30, 0.01, seed=4)
    d = _dev(rows, False)
    # beyond the array's size: refused with a message, nothing launched
    big = B.Replay(70_000, D, seed=1, max_append=4096, distinct=True)
    big.append(d["s"], d["s_next"], d["a"], d["r"], d["term"])
    out = big.alloc_batch(65_537)
    with pytest.raises(B.ReplayError, match="65536") as e:
        big.sample_gather_static(0, 65_537, out)
    assert e.value.status == B.RP_EINVAL
    assert big.sample_gather(0, 65_537)[0] == 0          # the allocating entry point takes it
    # burn-in and too few experiences are refused as by replay_sample_gather
    few = B.Replay(64, D, seed=1, burn_in=10, distinct=True)
    out = few.alloc_batch(8)
    assert few.sample_gather_static(0, 8, out)[0] == B.RP_SKIPPED_BURN_IN
    # sampling with replacement needs no scratch: same results, no batch limit of its own
    plain = B.Replay(70_000, D, seed=2, max_append=4096)
    plain.append(d["s"], d["s_next"], d["a"], d["r"], d["term"])
    for step, batch in [(0, 70_001), (1, 32)]:
        want = plain.sample_gather(step, batch)[1]
        st, got = plain.sample_gather_static(step, batch, plain.alloc_batch(batch))
        assert st == 0
        _same(got, want, "with replacement")
