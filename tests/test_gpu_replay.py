"""GPU parity of the replay entry points against the CPU oracle: bit-exact ring state,
sampled slot numbers and gathered batches, through the C ABI."""
import numpy as np
import pytest
import torch

import oracle
from paper_1801_03138_amd import synth

pytestmark = pytest.mark.gpu

DT = {"f32": (oracle.F32, 0), "bf16": (oracle.BF16, 1), "u8": (oracle.U8, 2)}


@pytest.fixture(scope="module")
def B():
    from paper_1801_03138_amd import binding
    assert torch.cuda.is_available(), "these tests need the MI355X"
    binding.lib()
    return binding


def _rows(n, D, A, p_term, seed, dtype):
    if dtype == "u8":
        fr = synth.frames(n, D, A, p_term, seed)
        fr["s_next"] = synth.frames(n, D, A, p_term, seed + 1000)["s"]
        return fr
    return synth.experiences(n, D, A, p_term, seed, state_dtype=dtype)


def _to_dev(part):
    return {k: (None if v is None else torch.from_numpy(np.ascontiguousarray(v).view(
        np.int16 if v.dtype == np.uint16 else v.dtype)).cuda()) for k, v in part.items()}


def _append_both(gpu, ref, part, device_src, chain=False):
    sn = None if chain else part["s_next"]
    ref.append(part["s"], sn, part["a"], part["r"], part["term"])
    if device_src:
        d = _to_dev(part)
        gpu.append(d["s"], None if chain else d["s_next"], d["a"], d["r"], d["term"])
        torch.cuda.synchronize()
    else:
        gpu.append(part["s"], sn, part["a"], part["r"], part["term"])


def _assert_ring_equal(gpu, ref):
    assert gpu.state() == ref.state()
    C = ref.capacity
    g = gpu.read_rows(0, C)
    o = ref.read(0, C)
    for x, y, name in zip(g, o, synth.FIELDS):
        if x is None:
            assert y is None
            continue
        assert np.array_equal(x.view(np.uint8), y.view(np.uint8)), name


def _assert_batch_equal(out, ref, idx):
    torch.cuda.synchronize()
    s, sn, a, r, t, gi = [x.cpu() for x in out]
    os_, osn, oa, or_, ot = ref.gather(idx)
    assert np.array_equal(gi.numpy().view(np.uint32), idx)

    def raw(x):
        return x.view(torch.int16).numpy() if x.dtype == torch.bfloat16 else x.numpy()
    assert np.array_equal(raw(s).view(np.uint8), os_.view(np.uint8))
    assert np.array_equal(raw(sn).view(np.uint8), osn.view(np.uint8))
    assert np.array_equal(a.numpy(), oa)
    assert np.array_equal(r.numpy().view(np.uint32), or_.view(np.uint32))
    assert np.array_equal(t.numpy(), ot)


@pytest.mark.parametrize("dtype", ["f32", "bf16", "u8"])
@pytest.mark.parametrize("device_src", [False, True])
def test_append_wraparound_matches_oracle(B, dtype, device_src):
    C, D = 1000, 27
    gpu = B.Replay(C, D, DT[dtype][1], B.RP_PAIR, max_append=300)
    ref = oracle.Ring(C, D, DT[dtype][0])
    rows = _rows(5000, D, 30, 0.05, 0, dtype)
    k = 0
    for n in [1, 1, 7, 300, 301, 390, 1, 999, 1000, 5, 640, 360, 64]:
        _append_both(gpu, ref, synth.take(rows, k, k + n), device_src)
        k += n
        _assert_ring_equal(gpu, ref)


@pytest.mark.parametrize("capacity", [1, 2, 3, 5])
def test_tiny_rings_every_append_size(B, capacity):
    D = 3
    rows = _rows(200, D, 4, 0.3, capacity, "f32")
    for n in range(1, capacity + 1):
        gpu = B.Replay(capacity, D, max_append=2)
        ref = oracle.Ring(capacity, D)
        k = 0
        for _ in range(2 * capacity + 1):
            _append_both(gpu, ref, synth.take(rows, k, k + n), False)
            k += n
            _assert_ring_equal(gpu, ref)
            idx = ref.sample(0, k, 9)
            st, out = gpu.sample_gather(k, 9)
            assert st == 0
            _assert_batch_equal(out, ref, idx)


@pytest.mark.parametrize("dtype,D", [("f32", 27), ("bf16", 27), ("u8", 27), ("f32", 1), ("f32", 64),
                                     ("bf16", 100), ("u8", 1001), ("f32", 500)])
def test_sample_gather_matches_oracle_while_filling(B, dtype, D):
    C = 777
    gpu = B.Replay(C, D, DT[dtype][1], B.RP_PAIR, seed=5, max_append=256)
    ref = oracle.Ring(C, D, DT[dtype][0])
    rows = _rows(2000, D, 30, 0.05, 1, dtype)
    k, step = 0, 0
    for n in [1, 2, 61, 200, 400, 113, 600]:
        _append_both(gpu, ref, synth.take(rows, k, k + n), True)
        k += n
        for batch in [1, 3, 16, 17, 128, 1000]:
            idx = ref.sample(5, step, batch)
            st, out = gpu.sample_gather(step, batch)
            assert st == 0
            assert idx.max() < ref.state()[1]
            _assert_batch_equal(out, ref, idx)
            step += 1


def test_special_bit_patterns_survive(B):
    bits = np.array([[0x7FC00001, 0x80000000, 0x00000001], [0xFFFFFFFF, 0x7F800000, 0x00400000]],
                    np.uint32)
    s = bits.view(np.float32)
    part = {"s": s, "s_next": s[::-1].copy(), "a": np.array([3, 2**24 + 1], np.int32),
            "r": bits[:, 0].view(np.float32).copy(), "term": np.array([0, 200], np.uint8)}
    gpu = B.Replay(2, 3)
    ref = oracle.Ring(2, 3)
    _append_both(gpu, ref, part, False)
    _assert_ring_equal(gpu, ref)
    st, out = gpu.sample_gather(0, 64)
    _assert_batch_equal(out, ref, ref.sample(0, 0, 64))


def test_u8_division_all_values(B):
    gpu = B.Replay(2, 256, B.RP_U8, B.RP_PAIR)
    ref = oracle.Ring(2, 256, oracle.U8)
    v = np.arange(256, dtype=np.uint8)[None, :]
    part = {"s": v, "s_next": v[:, ::-1].copy(), "a": [1], "r": [0.5], "term": [0]}
    _append_both(gpu, ref, part, False)
    st, out = gpu.sample_gather(0, 4)
    _assert_batch_equal(out, ref, ref.sample(0, 0, 4))
    chain = B.Replay(4, 256, B.RP_U8, B.RP_CHAIN)
    cref = oracle.Ring(4, 256, oracle.U8, oracle.CHAIN)
    part = {"s": np.concatenate([v, v[:, ::-1]]), "s_next": None, "a": [1, 2], "r": [0.5, 1.5],
            "term": [0, 1]}
    _append_both(chain, cref, part, False, chain=True)
    st, out = chain.sample_gather(3, 5)
    assert st == 0
    _assert_batch_equal(out, cref, cref.sample(0, 3, 5))


def test_burn_in_refuses_and_writes_nothing(B):
    gpu = B.Replay(64, 4, burn_in=10, seed=1)
    ref = oracle.Ring(64, 4, burn_in=10)
    rows = _rows(20, 4, 3, 0.1, 0, "f32")
    out = gpu.alloc_batch(8)
    for t in out:
        t.fill_(7)
    st, _ = gpu.sample_gather(0, 8, out=out)
    assert st == B.RP_SKIPPED_BURN_IN
    _append_both(gpu, ref, synth.take(rows, 0, 9), False)
    st, _ = gpu.sample_gather(0, 8, out=out)
    assert st == B.RP_SKIPPED_BURN_IN and ref.sample(1, 0, 8) is None
    torch.cuda.synchronize()
    assert all(bool((t == 7).all()) for t in out)
    _append_both(gpu, ref, synth.take(rows, 9, 10), False)
    st, out = gpu.sample_gather(0, 8, out=out)
    assert st == 0
    _assert_batch_equal(out, ref, ref.sample(1, 0, 8))


def test_error_paths(B):
    gpu = B.Replay(8, 2)
    rows = _rows(16, 2, 3, 0.1, 0, "f32")
    with pytest.raises(B.ReplayError) as e:
        gpu.append(rows["s"][:9], rows["s_next"][:9], rows["a"][:9], rows["r"][:9], rows["term"][:9])
    assert e.value.status == B.RP_EINVAL and "capacity" in str(e.value)
    assert gpu.state() == (0, 0, 0)
    gpu.append(rows["s"][:0], rows["s_next"][:0], rows["a"][:0], rows["r"][:0], rows["term"][:0])
    assert gpu.state() == (0, 0, 0)
    gpu.append(rows["s"][:3], rows["s_next"][:3], rows["a"][:3], rows["r"][:3], rows["term"][:3])
    with pytest.raises(B.ReplayError):
        gpu.sample_gather(0, 0)
    with pytest.raises(B.ReplayError):
        B.Replay(0, 2)
    with pytest.raises(B.ReplayError):
        B.Replay(8, 100000, B.RP_F32, B.RP_PAIR)  # packed row too large: use the CHAIN layout


@pytest.mark.parametrize("dtype,D", [("u8", 28224), ("u8", 37), ("u8", 4096), ("f32", 27),
                                     ("bf16", 27), ("f32", 1024), ("bf16", 4100)])
def test_chain_layout_matches_oracle(B, dtype, D):
    C = 41
    gpu = B.Replay(C, D, DT[dtype][1], B.RP_CHAIN, seed=2, max_append=16)
    ref = oracle.Ring(C, D, DT[dtype][0], oracle.CHAIN)
    rows = _rows(200, D, 18, 0.1, 3, dtype)
    k, step = 0, 0
    st, _ = gpu.sample_gather(0, 4)
    assert st == B.RP_SKIPPED_BURN_IN
    for n, dev in [(1, False), (1, True), (5, False), (30, True), (9, False), (41, True), (17, False)]:
        _append_both(gpu, ref, synth.take(rows, k, k + n), dev, chain=True)
        k += n
        _assert_ring_equal(gpu, ref)
        for batch in [1, 7, 32, 256]:
            idx = ref.sample(2, step, batch)
            st, out = gpu.sample_gather(step, batch)
            if idx is None:
                assert st == B.RP_SKIPPED_BURN_IN
                continue
            assert st == 0
            _assert_batch_equal(out, ref, idx)
            step += 1


def test_paper_shaped_ring_full_size(B):
    """Capacity 1,000,000 x (27+27+3) values, filled past the wrap point, batches up to 65,536."""
    C, D = 1_000_000, 27
    gpu = B.Replay(C, D, seed=0, max_append=4096)
    ref = oracle.Ring(C, D)
    rows = _rows(250_000, D, 30, 0.005, 0, "f32")
    for rep in range(5):          # 1.25 M appends: the ring wraps once
        for lo in range(0, 250_000, 62_500):
            part = synth.take(rows, lo, lo + 62_500)
            part["r"] = part["r"] + np.float32(rep)
            _append_both(gpu, ref, part, True)
    assert gpu.state() == ref.state() == (250_000, C, 1_250_000)
    probe = [0, 1, 249_999, 250_000, 999_999]
    for p in probe:
        g, o = gpu.read_rows(p, 1), ref.read(p, 1)
        assert all(np.array_equal(x.view(np.uint8), y.view(np.uint8)) for x, y in zip(g, o))
    # (from 32,769 rows on a thread of the gather takes two rows, from 65,537 four: ragged on both sides)
    for step, batch in enumerate([32, 128, 512, 2048, 8192, 32768, 32769, 65536, 65537, 150_001]):
        st, out = gpu.sample_gather(step, batch)
        assert st == 0
        _assert_batch_equal(out, ref, ref.sample(0, step, batch))


def test_large_state_ring_full_size(B):
    """200,000 slots of 84x84x4 bytes (5.6 GB), one state per experience, batches 32 and 256."""
    C, D = 200_000, 84 * 84 * 4
    gpu = B.Replay(C, D, B.RP_U8, B.RP_CHAIN, seed=3, max_append=64)
    ref = oracle.Ring(C, D, oracle.U8, oracle.CHAIN)
    total, chunk = 0, 10_000
    base = synth.frames(chunk, D, 18, 0.001, seed=11)
    while total < C + 30_000:       # wraps: the newest slot ends up in the middle of the ring
        part = dict(base)
        part["s"] = np.roll(base["s"], total // chunk, axis=1)   # a different chunk every time
        _append_both(gpu, ref, part, True, chain=True)
        total += chunk
    assert gpu.state() == ref.state()
    for step, batch in enumerate([32, 256, 32, 256]):
        st, out = gpu.sample_gather(step, batch)
        assert st == 0
        _assert_batch_equal(out, ref, ref.sample(3, step, batch))


@pytest.mark.parametrize("dtype,D,chain", [("f32", 27, False), ("bf16", 27, False), ("u8", 37, True)])
def test_sampling_without_duplicates_matches_oracle(B, dtype, D, chain):
    """RP_DISTINCT: bit-exact slot numbers and batches, no slot twice, refused while fewer
    experiences can be drawn than the batch asks for; whole-ring batches are permutations."""
    C = 300
    gpu = B.Replay(C, D, DT[dtype][1], B.RP_CHAIN if chain else B.RP_PAIR, seed=11, max_append=256,
                   distinct=True)
    ref = oracle.Ring(C, D, DT[dtype][0], oracle.CHAIN if chain else oracle.PAIR)
    rows = _rows(900, D, 30, 0.05, 2, dtype)
    k, step = 0, 0
    for n in [1, 2, 40, 100, 157, 250, 250]:
        _append_both(gpu, ref, synth.take(rows, k, k + n), True, chain=chain)
        k += n
        choices = ref.state()[1] - (1 if chain else 0)
        for batch in [1, 2, 16, 17, 64, 129, 299, 300]:
            idx = ref.sample(11, step, batch, distinct=True)
            st, out = gpu.sample_gather(step, batch)
            if batch > choices:
                assert idx is None and st == B.RP_SKIPPED_BURN_IN
                continue
            assert st == 0 and len(set(idx.tolist())) == batch
            _assert_batch_equal(out, ref, idx)
            if batch == choices:
                assert len(set(idx.tolist())) == choices
            step += 1


@pytest.mark.parametrize("chain", [False, True])
def test_sampling_without_duplicates_every_draw_shape(B, chain):
    """The kernel that draws a batch without duplicates gives a draw to a whole wavefront, to
    sixteen lanes or to one lane depending on the batch: batches on both sides of each limit
    (1,024 and 8,192), every slot number against the oracle, on a ring that has wrapped."""
    C, D = 20_000, 9
    gpu = B.Replay(C, D, DT["f32"][1], B.RP_CHAIN if chain else B.RP_PAIR, seed=21, max_append=4096,
                   distinct=True)
    ref = oracle.Ring(C, D, DT["f32"][0], oracle.CHAIN if chain else oracle.PAIR)
    rows = _rows(4000, D, 30, 0.05, 5, "f32")
    for k in range(7):                       # 28,000 experiences into 20,000 slots
        _append_both(gpu, ref, rows, True, chain=chain)
    for step, batch in enumerate([1024, 1025, 4096, 8192, 8193, 19_999]):
        idx = ref.sample(21, step, batch, distinct=True)
        st, out = gpu.sample_gather(step, batch)
        assert st == 0 and len(set(idx.tolist())) == batch
        _assert_batch_equal(out, ref, idx)


def test_sampling_without_duplicates_at_paper_size(B):
    """1,000,000 experiences, batch 65,536 and the smaller ones: the launch shapes the bench times;
    every slot number against the oracle on a sample of positions, all of them distinct."""
    C, D = 1_000_000, 27
    gpu = B.Replay(C, D, seed=3, max_append=4096, distinct=True)
    rows = synth.experiences(100_000, D, 30, 0.005, seed=0)
    d = _to_dev(rows)
    for _ in range(10):
        gpu.append(d["s"], d["s_next"], d["a"], d["r"], d["term"])
    st, out = gpu.sample_gather(7, 65536)
    assert st == 0
    torch.cuda.synchronize()
    idx = out[5].cpu().numpy().view(np.uint32)
    assert idx.max() < C and len(np.unique(idx)) == 65536
    for i in list(range(0, 65536, 997)) + [65535]:
        assert idx[i] == oracle.distinct_index(3, 7, i, C)
    # the gathered rows are those slots' rows (the ring holds the 100,000 source rows ten times)
    s = out[0].cpu().numpy()
    assert np.array_equal(s.view(np.uint32), rows["s"][idx % 100_000].view(np.uint32))
    # the smaller batches the bench times, which draw inside the gather's launch
    for step, batch in ((8, 128), (9, 2048), (10, 8192)):
        st, out = gpu.sample_gather(step, batch)
        assert st == 0
        torch.cuda.synchronize()
        idx = out[5].cpu().numpy().view(np.uint32)
        assert len(np.unique(idx)) == batch
        for i in list(range(0, batch, 61)) + [batch - 1]:
            assert idx[i] == oracle.distinct_index(3, step, i, C)
        s, sn = out[0].cpu().numpy(), out[1].cpu().numpy()
        assert np.array_equal(s.view(np.uint32), rows["s"][idx % 100_000].view(np.uint32))
        assert np.array_equal(sn.view(np.uint32), rows["s_next"][idx % 100_000].view(np.uint32))


def _random_rings(n, seed):
    rng = np.random.default_rng(seed)
    out = []
    for _ in range(n):
        dtype = str(rng.choice(["f32", "bf16", "u8"]))
        chain = bool(rng.random() < 0.4)
        D = int(rng.choice([1, 2, 3, 7, 27, 31, 32, 33, 63, 64, 65, 100, 255, 1000, 4099]))
        if not chain:
            D = min(D, 255)
        out.append(dict(dtype=dtype, chain=chain, D=D, capacity=int(rng.choice([1, 2, 7, 64, 129, 1000, 4097])),
                        burn_in=int(rng.choice([0, 0, 5, 50])), distinct=bool(rng.random() < 0.3),
                        seed=int(rng.integers(0, 10_000))))
    return out


@pytest.mark.parametrize("c", _random_rings(40, 271127), ids=lambda c: "%s-%s-D%d-C%d-%s" % (
    c["dtype"], "chain" if c["chain"] else "pair", c["D"], c["capacity"], "distinct" if c["distinct"] else "repl"))
def test_random_rings(B, c):
    """Seeded random rings: a run of appends of random sizes (host and device sources, wrapping
    several times) with sampling at random batch sizes in between; ring contents, state, slot
    numbers and batches bit-exact, refusals in the same places."""
    rng = np.random.default_rng(c["seed"])
    C, D, chain = c["capacity"], c["D"], c["chain"]
    gpu = B.Replay(C, D, DT[c["dtype"]][1], B.RP_CHAIN if chain else B.RP_PAIR, burn_in=c["burn_in"],
                   seed=c["seed"], max_append=min(C, 600), distinct=c["distinct"])
    ref = oracle.Ring(C, D, DT[c["dtype"]][0], oracle.CHAIN if chain else oracle.PAIR, burn_in=c["burn_in"])
    total = min(3 * C + 40, 2500 if D > 300 else 9000)
    rows = _rows(total, D, 11, 0.1, c["seed"], c["dtype"])
    k, step = 0, 0
    while k < total:
        n = int(min(total - k, min(C, 600), rng.choice([1, 1, 2, 3, 17, 64, 200, 600])))
        _append_both(gpu, ref, synth.take(rows, k, k + n), bool(rng.random() < 0.5), chain=chain)
        k += n
        for batch in rng.choice([1, 2, 15, 16, 17, 100, 256, 1000], size=2):
            batch = int(batch)
            idx = ref.sample(c["seed"], step, batch, distinct=c["distinct"])
            st, out = gpu.sample_gather(step, batch)
            if idx is None:
                assert st == B.RP_SKIPPED_BURN_IN
                continue
            assert st == 0
            _assert_batch_equal(out, ref, idx)
            step += 1
    _assert_ring_equal(gpu, ref)
