"""Pins for the exact parts of the CPU oracle: FIFO ring, Philox sampling, gather/unpack.

Each test checks the oracle against something other than itself: a library
container, published known-answer vectors, closed forms, exact rational
arithmetic, or exhaustive enumeration on tiny rings.
"""
import collections
import math
import os
from fractions import Fraction

import numpy as np
import pytest

import oracle
from paper_1801_03138_amd import synth


def _paper_values(golden_dir):
    vals = {}
    with open(os.path.join(golden_dir, "paper_values.txt")) as f:
        for line in f:
            line = line.split("#")[0].strip()
            if line:
                k, v = line.split("=")
                vals[k.strip()] = float(v)
    return vals


# ----------------------------------------------------------------------------- Philox
def test_philox_known_answers(golden_dir):
    n = 0
    with open(os.path.join(golden_dir, "philox4x32_10_kat.txt")) as f:
        for line in f:
            if line.startswith("#") or not line.strip():
                continue
            w = [int(x, 16) for x in line.split()]
            got = oracle.philox4x32_10(w[0:4], w[4:6])
            assert [int(x) for x in got] == w[6:10]
            n += 1
    assert n == 3


def test_philox_is_a_bijection_of_the_counter():
    # a counter-based generator permutes counter space: distinct counters give distinct blocks
    seen = set()
    for c0 in range(64):
        for c2 in range(8):
            seen.add(tuple(int(x) for x in oracle.philox4x32_10([c0, 0, c2, 0], [7, 9])))
    assert len(seen) == 64 * 8


# ----------------------------------------------------------------------------- FIFO ring
def _tuple_rows(rows, k):
    return (rows["s"][k].tobytes(), rows["s_next"][k].tobytes(), int(rows["a"][k]),
            rows["r"][k].tobytes(), int(rows["term"][k]))


def _ring_logical(ring):
    """Ring content as a list of tuples from oldest to newest."""
    head, size, total = ring.state()
    first = (head - size) % ring.capacity
    s, sn, a, r, t = ring.read(first, size)
    return [(s[k].tobytes(), sn[k].tobytes(), int(a[k]), r[k].tobytes(), int(t[k]))
            for k in range(size)]


@pytest.mark.parametrize("capacity", [1, 2, 3, 4, 5])
def test_ring_matches_deque_for_every_append_sequence(capacity):
    """Every sequence of batched appends with sizes 1..C up to 4C experiences in total."""
    D = 2
    rows = synth.experiences(4 * capacity + capacity, D, 5, 0.3, seed=capacity)

    def explore(sizes_so_far, used):
        ring = oracle.Ring(capacity, D)
        dq = collections.deque(maxlen=capacity)
        k = 0
        for n in sizes_so_far:
            part = synth.take(rows, k, k + n)
            ring.append(part["s"], part["s_next"], part["a"], part["r"], part["term"])
            for j in range(k, k + n):
                dq.append(_tuple_rows(rows, j))
            k += n
            head, size, total = ring.state()
            assert total == k and size == min(k, capacity) and head == k % capacity
            assert _ring_logical(ring) == list(dq)
        if used < 4 * capacity and len(sizes_so_far) < 6:
            for n in range(1, capacity + 1):
                explore(sizes_so_far + [n], used + n)

    explore([], 0)


def test_ring_zero_append_and_oversize_append():
    ring = oracle.Ring(4, 3)
    rows = synth.experiences(8, 3, 4, 0.5, seed=1)
    ring.append(rows["s"][:0], rows["s_next"][:0], rows["a"][:0], rows["r"][:0], rows["term"][:0])
    assert ring.state() == (0, 0, 0)
    with pytest.raises(ValueError):
        ring.append(rows["s"][:5], rows["s_next"][:5], rows["a"][:5], rows["r"][:5],
                    rows["term"][:5])
    assert ring.state() == (0, 0, 0)


def test_tiny_config_wraps_four_times():
    """4096 single appends into capacity 1024: the ring holds rows 3072..4095 in slot order."""
    C, N, D = 1024, 4096, 27
    rows = synth.experiences(N, D, 8, 0.01, seed=0)
    ring = oracle.Ring(C, D)
    for k in range(N):
        p = synth.take(rows, k, k + 1)
        ring.append(p["s"], p["s_next"], p["a"], p["r"], p["term"])
    assert ring.state() == (0, C, N)
    s, sn, a, r, t = ring.read(0, C)
    assert np.array_equal(s.view(np.uint32), rows["s"][3072:].view(np.uint32))
    assert np.array_equal(sn.view(np.uint32), rows["s_next"][3072:].view(np.uint32))
    assert np.array_equal(a, rows["a"][3072:])
    assert np.array_equal(r.view(np.uint32), rows["r"][3072:].view(np.uint32))
    assert np.array_equal(t, rows["term"][3072:])


def test_terminal_is_normalised_to_zero_or_one():
    ring = oracle.Ring(4, 1)
    ring.append(np.zeros((3, 1), np.float32), np.zeros((3, 1), np.float32), [0, 1, 2], [0, 0, 0],
                np.array([0, 7, 255], np.uint8))
    assert list(ring.read(0, 3)[4]) == [0, 1, 1]


def test_row_width_matches_paper(golden_dir):
    pv = _paper_values(golden_dir)
    D = int(pv["state_floats"])
    assert 2 * D + 3 == pv["row_values"]
    assert 84 * 84 * 4 == pv["pixel_state_values"]
    assert 2 * int(pv["pixel_state_values"]) + 3 == pv["pixel_row_values"]


# ----------------------------------------------------------------------------- sampling
def test_indices_stay_in_range_at_every_fill_level():
    for size in [1, 2, 3, 5, 31, 32, 33, 1000, 4097, 10**6, 2**32 - 1]:
        idx = oracle.uniform_indices(3, 11, 4, 37, size)
        assert idx.max() < size
    assert not oracle.uniform_indices(3, 11, 4, 37, 1).any()


def test_power_of_two_size_takes_the_top_bits():
    seed, step = 5, 77
    for i in range(19):
        block = oracle.philox4x32_10([i // 4, 0, step, 0], [seed, 0])
        x = int(block[i % 4])
        for k in (1, 4, 10, 31):
            assert oracle.uniform_index(seed, step, i, 1 << k) == x >> (32 - k)


def test_seed_and_step_words():
    """Seed and step are 64-bit: low words feed key0 / counter word 2, high words key1 / word 3."""
    seed = (0xABCD << 32) | 0x1234
    step = (0x77 << 32) | 0x42
    for i in (0, 1, 2, 3, 4, 9):
        block = oracle.philox4x32_10([i // 4, 0, 0x42, 0x77], [0x1234, 0xABCD])
        assert oracle.uniform_index(seed, step, i, 2**32) == int(block[i % 4])


def test_sampling_is_reproducible_and_step_dependent():
    a = oracle.uniform_indices(0, 10, 3, 128, 10**6)
    b = oracle.uniform_indices(0, 10, 3, 128, 10**6)
    assert np.array_equal(a, b)
    assert not np.array_equal(a[0], a[1])
    assert not np.array_equal(a[0], oracle.uniform_indices(1, 10, 1, 128, 10**6)[0])
    # batch size does not change the earlier draws of a step
    assert np.array_equal(oracle.uniform_indices(0, 10, 1, 7, 10**6)[0], a[0][:7])


def test_chi_square_uniformity():
    """1,024,000 draws into 1024 bins; chi-square has 1023 degrees of freedom."""
    bins = 1024
    idx = oracle.uniform_indices(0, 0, 4000, 256, bins)
    counts = np.bincount(idx.ravel(), minlength=bins).astype(np.float64)
    expected = idx.size / bins
    chi2 = float(((counts - expected) ** 2 / expected).sum())
    assert abs(chi2 - 1023) < 5 * math.sqrt(2 * 1023), chi2


def test_chi_square_uniformity_non_power_of_two():
    bins = 1000
    idx = oracle.uniform_indices(9, 5, 4000, 250, bins)
    counts = np.bincount(idx.ravel(), minlength=bins).astype(np.float64)
    expected = idx.size / bins
    chi2 = float(((counts - expected) ** 2 / expected).sum())
    assert abs(chi2 - 999) < 5 * math.sqrt(2 * 999), chi2


def test_draws_within_a_batch_are_independent():
    """Pairs (draw i, draw i+1) of the same step fill a 16x16 table uniformly (df = 255)."""
    idx = oracle.uniform_indices(2, 0, 20000, 8, 16).astype(np.int64)
    pair = (idx[:, 0::2] * 16 + idx[:, 1::2]).ravel()
    counts = np.bincount(pair, minlength=256).astype(np.float64)
    expected = pair.size / 256
    chi2 = float(((counts - expected) ** 2 / expected).sum())
    assert abs(chi2 - 255) < 5 * math.sqrt(2 * 255), chi2


def test_duplicate_rate_matches_the_paper(golden_dir):
    """The paper: a sample of 32 out of 1,000,000 repeats an experience 0.05% of the time."""
    pv = _paper_values(golden_dir)
    N, B = int(pv["replay_capacity"]), 32
    exact = 1.0 - math.prod(1.0 - k / N for k in range(B))
    assert round(100 * exact, 2) == pv["duplicate_rate_b32_percent"]
    batches, dup = 2_000_000, 0
    for c in range(0, batches, 250_000):
        idx = np.sort(oracle.uniform_indices(0, c, 250_000, B, N), axis=1)
        dup += int((idx[:, 1:] == idx[:, :-1]).any(axis=1).sum())
    expect = exact * batches
    assert abs(dup - expect) < 5 * math.sqrt(expect), (dup, expect)


def test_no_sampling_during_burn_in():
    ring = oracle.Ring(16, 2, burn_in=5)
    rows = synth.experiences(8, 2, 3, 0.1, seed=2)
    assert ring.sample(0, 0, 4) is None  # empty
    for k in range(4):
        p = synth.take(rows, k, k + 1)
        ring.append(p["s"], p["s_next"], p["a"], p["r"], p["term"])
        assert ring.sample(0, 0, 4) is None
    p = synth.take(rows, 4, 5)
    ring.append(p["s"], p["s_next"], p["a"], p["r"], p["term"])
    idx = ring.sample(0, 0, 64)
    assert idx is not None and idx.max() < 5


def test_empty_ring_without_burn_in_refuses():
    assert oracle.Ring(4, 1).sample(0, 0, 2) is None
    chain = oracle.Ring(4, 1, oracle.U8, oracle.CHAIN)
    chain.append(np.zeros((1, 1), np.uint8), None, [0], [0.0], [0])
    assert chain.sample(0, 0, 2) is None  # a single state has no successor


# ----------------------------------------------------------------------------- gather
def _seq_rows(first, n, D):
    """Experiences whose every field encodes the global sequence number."""
    k = np.arange(first, first + n)
    s = np.repeat(k[:, None], D, axis=1).astype(np.float32) + np.arange(D, dtype=np.float32) / 64
    return {"s": s, "s_next": -s, "a": k.astype(np.int32), "r": (k * 0.5).astype(np.float32),
            "term": (k % 3 == 0).astype(np.uint8)}


def test_gather_round_trip_property():
    """Sampled rows decode to a sequence number that lives in the sampled slot and is still retained."""
    C, D = 97, 3
    ring = oracle.Ring(C, D)
    total = 0
    for n in [5, 40, 60, 1, 97, 13]:
        p = _seq_rows(total, n, D)
        ring.append(p["s"], p["s_next"], p["a"], p["r"], p["term"])
        total += n
        head, size, tot = ring.state()
        idx = ring.sample(4, total, 256)
        s, sn, a, r, t = ring.gather(idx)
        seq = a.astype(np.int64)
        assert np.all(seq % C == idx)
        assert np.all(seq >= tot - size) and np.all(seq < tot)
        assert np.array_equal(s[:, 0], seq.astype(np.float32))
        assert np.array_equal(sn, -s)
        assert np.array_equal(r, (seq * 0.5).astype(np.float32))
        assert np.array_equal(t, (seq % 3 == 0).astype(np.uint8))


def test_gather_enumerates_every_slot_on_tiny_rings():
    for C in (1, 2, 3, 7):
        D = 4
        rows = synth.experiences(2 * C + 1, D, 9, 0.5, seed=C)
        ring = oracle.Ring(C, D)
        ring.append(*[synth.take(rows, 0, C)[f] for f in synth.FIELDS])
        for j in range(C, 2 * C + 1):
            ring.append(*[synth.take(rows, j, j + 1)[f] for f in synth.FIELDS])
        newest_first = 2 * C + 1 - C
        for slot in range(C):
            # the experience in `slot` is the latest k with k mod C == slot
            k = max(j for j in range(2 * C + 1) if j % C == slot)
            assert k >= newest_first
            s, sn, a, r, t = ring.gather([slot])
            assert s.tobytes() == rows["s"][k].tobytes()
            assert sn.tobytes() == rows["s_next"][k].tobytes()
            assert a[0] == rows["a"][k] and t[0] == rows["term"][k]
            assert r.tobytes() == rows["r"][k].tobytes()


def test_gather_preserves_special_bit_patterns():
    """A pure copy: NaN payloads, negative zero and denormals survive bit for bit."""
    bits = np.array([[0x7FC00001, 0x80000000, 0x00000001], [0xFFFFFFFF, 0x7F800000, 0x00400000]],
                    np.uint32)
    s = bits.view(np.float32)
    ring = oracle.Ring(2, 3)
    ring.append(s, s[::-1].copy(), [3, 2**24 + 1], bits[:, 0].view(np.float32), [0, 1])
    gs, gsn, a, r, t = ring.gather([1, 0, 1])
    assert np.array_equal(gs.view(np.uint32), bits[[1, 0, 1]])
    assert np.array_equal(gsn.view(np.uint32), bits[::-1][[1, 0, 1]])
    assert list(a) == [2**24 + 1, 3, 2**24 + 1]
    assert np.array_equal(r.view(np.uint32), bits[[1, 0, 1], 0])


def test_bf16_states_are_copied_verbatim():
    rows = synth.experiences(10, 5, 4, 0.2, seed=3, state_dtype="bf16")
    ring = oracle.Ring(8, 5, oracle.BF16)
    ring.append(rows["s"][:8], rows["s_next"][:8], rows["a"][:8], rows["r"][:8], rows["term"][:8])
    ring.append(rows["s"][8:], rows["s_next"][8:], rows["a"][8:], rows["r"][8:], rows["term"][8:])
    s, sn, a, r, t = ring.gather([0, 1, 2])
    assert s.dtype == np.uint16
    assert np.array_equal(s, rows["s"][[8, 9, 2]]) and np.array_equal(sn, rows["s_next"][[8, 9, 2]])


def test_u8_to_float_is_correctly_rounded_division():
    """float(u8)/255 must be the float32 nearest to the rational k/255 for all 256 values."""
    ring = oracle.Ring(1, 256, oracle.U8, oracle.PAIR)
    vals = np.arange(256, dtype=np.uint8)[None, :]
    ring.append(vals, vals[:, ::-1].copy(), [0], [0.0], [0])
    s, sn, *_ = ring.gather([0])
    assert s.dtype == np.float32
    for k in range(256):
        f = np.float32(s[0, k])
        exact = Fraction(k, 255)
        err = abs(Fraction(float(f)) - exact)
        for nb in (np.nextafter(f, np.float32(2)), np.nextafter(f, np.float32(-1))):
            assert err <= abs(Fraction(float(nb)) - exact)
        assert sn[0, 255 - k] == f
    assert s[0, 0] == 0.0 and s[0, 255] == 1.0 and s[0, 51] == np.float32(0.2)


def test_chain_layout_next_state_is_next_slot():
    """One state per experience (Discussion): s' of slot p is the state stored in slot p+1."""
    C, D = 6, 5
    fr = synth.frames(9, D, 4, 0.3, seed=5)
    ring = oracle.Ring(C, D, oracle.U8, oracle.CHAIN)
    ring.append(fr["s"][:4], None, fr["a"][:4], fr["r"][:4], fr["term"][:4])
    # 4 states stored: experiences 0,1,2 are complete, 3 (newest) has no successor
    hits = set()
    for step in range(200):
        idx = ring.sample(1, step, 8)
        hits.update(int(i) for i in idx)
    assert hits == {0, 1, 2}
    ring.append(fr["s"][4:], None, fr["a"][4:], fr["r"][4:], fr["term"][4:])
    head, size, total = ring.state()
    assert (head, size, total) == (3, 6, 9)
    newest_slot = (head - 1) % C
    hits = set()
    for step in range(400):
        idx = ring.sample(1, step, 8)
        hits.update(int(i) for i in idx)
        s, sn, a, r, t = ring.gather(idx)
        for j, p in enumerate(idx):
            k = max(q for q in range(9) if q % C == p)     # experience stored in slot p
            assert np.array_equal(s[j], fr["s"][k].astype(np.float32) / np.float32(255))
            assert np.array_equal(sn[j], fr["s"][k + 1].astype(np.float32) / np.float32(255))
            assert a[j] == fr["a"][k] and t[j] == fr["term"][k]
    assert hits == set(range(C)) - {newest_slot}


def test_chain_sampling_is_uniform_over_complete_experiences():
    C = 64
    ring = oracle.Ring(C, 1, oracle.U8, oracle.CHAIN)
    fr = synth.frames(C + 10, 1, 2, 0.0, seed=1)
    ring.append(fr["s"][:C], None, fr["a"][:C], fr["r"][:C], fr["term"][:C])
    ring.append(fr["s"][C:], None, fr["a"][C:], fr["r"][C:], fr["term"][C:])
    counts = np.zeros(C)
    for step in range(500):
        counts += np.bincount(ring.sample(7, step, 126), minlength=C)
    newest = (ring.state()[0] - 1) % C
    assert counts[newest] == 0
    others = np.delete(counts, newest)
    expected = 500 * 126 / (C - 1)
    chi2 = float(((others - expected) ** 2 / expected).sum())
    assert abs(chi2 - (C - 2)) < 5 * math.sqrt(2 * (C - 2)), chi2


# ---------------------------------------------------------------- sampling without duplicates
def test_distinct_sample_is_a_permutation_of_the_choices():
    """Fed with 0..n-1 the generator must return every choice exactly once, for every n."""
    for n in list(range(1, 70)) + [255, 256, 257, 1000, 4096, 4097]:
        for seed, step in ((0, 0), (7, 3), (2**40 + 5, 2**33 + 1)):
            out = oracle.distinct_indices(seed, step, n, n)
            assert sorted(out.tolist()) == list(range(n)), (n, seed, step)


def test_distinct_sample_at_paper_size_has_no_duplicates():
    """With replacement a batch of 32 out of 1,000,000 repeats an experience 0.05 % of the time
    (Methods); without, never."""
    for step in range(300):
        idx = oracle.distinct_indices(0, step, 32, 1_000_000)
        assert idx.max() < 1_000_000 and len(set(idx.tolist())) == 32
    big = oracle.distinct_indices(1, 0, 20_000, 1_000_000)
    assert len(set(big.tolist())) == 20_000


def test_distinct_sample_is_uniform_and_changes_with_the_step():
    # chi-square of the first member over 1000 choices, 100,000 steps: df = 999
    n, steps = 1000, 100_000
    first = np.array([oracle.distinct_index(5, k, 0, n) for k in range(steps)])
    counts = np.bincount(first, minlength=n)
    chi2 = ((counts - steps / n) ** 2 / (steps / n)).sum()
    assert abs(chi2 - 999) < 5 * np.sqrt(2 * 999)
    # ordered pairs (member 0, member 1) over 6 choices: 30 equally likely outcomes, df = 29
    pairs = np.zeros((6, 6))
    for k in range(30_000):
        a, b = oracle.distinct_index(9, k, 0, 6), oracle.distinct_index(9, k, 1, 6)
        assert a != b
        pairs[a, b] += 1
    exp = 30_000 / 30
    chi2 = ((pairs[~np.eye(6, dtype=bool)] - exp) ** 2 / exp).sum()
    assert abs(chi2 - 29) < 5 * np.sqrt(2 * 29)
    # whole samples of 5 out of 5: all 120 orders equally likely, df = 119 (a keyed permutation
    # built from too few or too regular rounds reaches only part of them)
    orders = {}
    for k in range(60_000):
        o = tuple(oracle.distinct_indices(3, k, 5, 5).tolist())
        orders[o] = orders.get(o, 0) + 1
    assert len(orders) == 120
    chi2 = sum((c - 500.0) ** 2 / 500.0 for c in orders.values())
    assert abs(chi2 - 119) < 5 * np.sqrt(2 * 119)
    # the key is (seed, step): other steps and seeds give other samples, the same ones the same
    a = oracle.distinct_indices(3, 10, 64, 10_000)
    assert np.array_equal(a, oracle.distinct_indices(3, 10, 64, 10_000))
    assert not np.array_equal(a, oracle.distinct_indices(3, 11, 64, 10_000))
    assert not np.array_equal(a, oracle.distinct_indices(4, 10, 64, 10_000))


def test_ring_sampling_without_duplicates():
    ring = oracle.Ring(50, 3, burn_in=0)
    rows = synth.experiences(40, 3, 4, 0.1, seed=1)
    ring.append(rows["s"][:10], rows["s_next"][:10], rows["a"][:10], rows["r"][:10], rows["term"][:10])
    assert ring.sample(0, 0, 11, distinct=True) is None          # only 10 to choose from
    idx = ring.sample(0, 0, 10, distinct=True)
    assert sorted(idx.tolist()) == list(range(10))
    chain = oracle.Ring(8, 3, oracle.F32, oracle.CHAIN, burn_in=0)
    for lo in range(0, 12, 4):
        chain.append(rows["s"][lo:lo + 4], None, rows["a"][lo:lo + 4], rows["r"][lo:lo + 4],
                     rows["term"][lo:lo + 4])
    # full ring of 8 with head 4: the newest slot (3) has no successor and is never drawn
    assert chain.sample(0, 0, 8, distinct=True) is None
    assert sorted(chain.sample(0, 1, 7, distinct=True).tolist()) == [0, 1, 2, 4, 5, 6, 7]
