"""Pins for the oracle's random numbers and sampler (CPU only).

The sampler's exact ids are defined by the oracle itself; what is checked here is
everything the paper and the mathematics fix: the published Philox vectors, an independent
big-integer Philox, Floyd's subset properties and uniformity, and the structure of a
GraphSAGE-style sample (Section 2.1 "Neighborhood Sampling", Section 3.1 "Superbatch
Sample").
"""
import os

import numpy as np
import pytest

import oracle
from workload import make_workload

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")
M32 = 0xFFFFFFFF


def philox_bigint(ctr, key, rounds=10):
    """Independent Philox4x32 written with Python integers from the SC'11 definition."""
    c = list(ctr)
    k = list(key)
    for _ in range(rounds):
        hi0, lo0 = divmod(0xD2511F53 * c[0], 1 << 32)
        hi1, lo1 = divmod(0xCD9E8D57 * c[2], 1 << 32)
        c = [hi1 ^ c[1] ^ k[0], lo1, hi0 ^ c[3] ^ k[1], lo0]
        k = [(k[0] + 0x9E3779B9) & M32, (k[1] + 0xBB67AE85) & M32]
    return c


def test_philox_known_answers():
    rows = [l.split() for l in open(os.path.join(GOLDEN, "philox4x32_10_kat.txt"))
            if l.strip() and not l.startswith("#")]
    assert len(rows) == 3
    for r in rows:
        v = [int(x, 16) for x in r]
        got = oracle.philox4x32_10(v[0:4], v[4:6])
        assert [int(x) for x in got] == v[6:10]
        assert philox_bigint(v[0:4], v[4:6]) == v[6:10]


def test_philox_matches_bigint_on_random_blocks():
    rng = np.random.default_rng(1)
    blocks = rng.integers(0, 1 << 32, size=(20000, 6), dtype=np.uint64)
    for row in blocks:
        row = [int(x) for x in row]
        assert [int(x) for x in oracle.philox4x32_10(row[:4], row[4:])] == \
            philox_bigint(row[:4], row[4:])


def test_philox_is_injective_on_a_counter_sweep():
    outs = set()
    for n in range(4096):
        outs.add(tuple(int(x) for x in oracle.philox4x32_10([n, 7, 1, n & 3], [5, 9])))
    assert len(outs) == 4096


def test_draw64_takes_words_1_and_0_of_the_block():
    seed = 0x1234567890ABCDEF
    x = philox_bigint([11, 22, 2, 5], [seed & M32, seed >> 32])
    assert oracle.draw64(seed, 11, 22, 2, 5) == (x[1] << 32) | x[0]


def floyd_reference(seed, node, batch, hop, deg, k):
    """Floyd's subset algorithm retyped with Python integers and the big-int Philox."""
    if deg <= k:
        return list(range(deg))
    chosen = []
    for i in range(k):
        j = deg - k + i
        x = philox_bigint([node, batch, hop, i], [seed & M32, seed >> 32])
        t = (((x[1] << 32) | x[0]) * (j + 1)) >> 64
        chosen.append(j if t in chosen else t)
    return sorted(chosen)


@pytest.mark.parametrize("deg", [0, 1, 9, 10, 11, 12, 64, 5641, (1 << 40) + 3])
def test_floyd_count_range_distinct(deg):
    for node in range(50):
        p = oracle.floyd_picks(3, node, 4, 1, deg, 10)
        assert len(p) == min(deg, 10)
        assert len(set(p.tolist())) == len(p)
        assert all(0 <= x < deg for x in p)
        assert list(p) == sorted(p)
        assert list(p) == floyd_reference(3, node, 4, 1, deg, 10)
        if deg <= 10:
            assert list(p) == list(range(deg))


@pytest.mark.parametrize("deg", [11, 12, 64])
def test_floyd_membership_is_uniform(deg):
    # every position must be picked with probability k/deg; chi-square over positions
    k, trials = 10, 60000
    hits = np.zeros(deg)
    for node in range(trials):
        hits[oracle.floyd_picks(0, node, 0, 0, deg, k)] += 1
    expect = trials * k / deg
    chi2 = ((hits - expect) ** 2 / expect).sum() * deg / (deg - k)  # finite-population factor
    # deg-1 degrees of freedom; 99.99th percentile of chi2(63) is ~118, of chi2(10) ~ 36
    assert chi2 < {11: 40, 12: 42, 64: 125}[deg]
    # pairs: positions (0,1) picked together with probability k(k-1)/(deg(deg-1))
    both = sum(1 for node in range(20000)
               if {0, 1} <= set(oracle.floyd_picks(0, node, 1, 0, deg, k).tolist()))
    p = k * (k - 1) / (deg * (deg - 1))
    assert abs(both - 20000 * p) < 5 * np.sqrt(20000 * p * (1 - p)) + 1


@pytest.fixture(scope="module")
def tiny():
    w = make_workload(1, features=False)
    r = oracle.sample_superbatch(w.offsets.numpy(), w.indices.numpy(), w.seeds.numpy(),
                                 w.seed_offsets.numpy(), w.cfg.fanout, rng_seed=0)
    return w, r


def check_sample_structure(offsets, indices, seeds, seed_offsets, fanout, r):
    S, H = len(seed_offsets) - 1, len(fanout)
    for b in range(S):
        ids = r["ids"][r["ids_offsets"][b]:r["ids_offsets"][b + 1]]
        sd = seeds[seed_offsets[b]:seed_offsets[b + 1]]
        hs = r["hop_sizes"][b]
        assert len(set(ids.tolist())) == len(ids)          # ids are distinct
        assert np.array_equal(ids[:len(sd)], sd)            # the list starts with the seeds
        assert hs[0] == len(sd) and hs[-1] == len(ids)
        assert all(hs[h] <= hs[h + 1] for h in range(H))
        for h in range(H):
            g = b * H + h
            rp = r["adj_rowptr"][r["adj_row_offsets"][g]:r["adj_row_offsets"][g + 1]]
            col = r["adj_col"][r["adj_col_offsets"][g]:r["adj_col_offsets"][g + 1]]
            assert len(rp) == hs[h] + 1 and rp[0] == 0 and rp[-1] == len(col)
            first_seen = hs[h]
            for row in range(hs[h]):
                v = ids[row]
                picks = col[rp[row]:rp[row + 1]]
                lo, hi = offsets[v], offsets[v + 1]
                assert len(picks) == min(hi - lo, fanout[h])        # "at most k", all if fewer
                nbrs = indices[lo:hi]
                assert all(c < hs[h + 1] for c in picks)
                # every pick is a neighbour of v, with the right multiplicity
                got = np.sort(ids[picks])
                pos = oracle.floyd_picks(0, int(v), b, h, int(hi - lo), fanout[h])
                assert np.array_equal(got, np.sort(nbrs[pos]))
                # new ids are appended in the order they are first met
                for c in picks:
                    if c >= first_seen:
                        assert c == first_seen
                        first_seen += 1
            assert first_seen == hs[h + 1]


def test_sample_structure_on_tiny_config(tiny):
    w, r = tiny
    check_sample_structure(w.offsets.numpy(), w.indices.numpy(), w.seeds.numpy(),
                           w.seed_offsets.numpy(), w.cfg.fanout, r)
    # sizes in the range the paper quotes scale with the batch: 3 hops of fanout 10
    # cannot exceed batch * 11**3 ids
    for b in range(w.cfg.S):
        n_seed = int(w.seed_offsets[b + 1] - w.seed_offsets[b])
        assert r["hop_sizes"][b][-1] <= n_seed * 11 ** 3


def test_fanout_3_2_single_seed_shape():
    # caption of the sampling figure: sampling size (3, 2), batch size 1
    w = make_workload(1, features=False)
    off, ind = w.offsets.numpy(), w.indices.numpy()
    deg = off[1:] - off[:-1]
    seed = int(np.argmax(deg >= 5))
    r = oracle.sample_superbatch(off, ind, [seed], [0, 1], [3, 2])
    hs = r["hop_sizes"][0]
    assert hs[0] == 1 and hs[1] <= 1 + 3 and hs[2] <= hs[1] + 2 * hs[1]
    rp0 = r["adj_rowptr"][r["adj_row_offsets"][0]:r["adj_row_offsets"][1]]
    assert list(rp0) == [0, 3]
    rp1 = r["adj_rowptr"][r["adj_row_offsets"][1]:r["adj_row_offsets"][2]]
    assert all(0 <= d <= 2 for d in np.diff(rp1))
    check_sample_structure(off, ind, np.array([seed], dtype=np.int32), np.array([0, 1]),
                           [3, 2], r)


def test_batch_result_does_not_depend_on_superbatch_partition(tiny):
    # Section 3.1 "Implications on Training Quality": the schedule only reorders
    # independent work, so batch b must come out the same whichever superbatch holds it
    w, r = tiny
    off, ind = w.offsets.numpy(), w.indices.numpy()
    so = w.seed_offsets.numpy()
    for lo, hi in [(0, 3), (3, 8), (5, 6)]:
        part = oracle.sample_superbatch(off, ind, w.seeds.numpy()[so[lo]:so[hi]],
                                        so[lo:hi + 1] - so[lo], w.cfg.fanout,
                                        rng_seed=0, first_batch_index=lo)
        for b in range(lo, hi):
            a = r["ids"][r["ids_offsets"][b]:r["ids_offsets"][b + 1]]
            c = part["ids"][part["ids_offsets"][b - lo]:part["ids_offsets"][b - lo + 1]]
            assert np.array_equal(a, c)
    other = oracle.sample_superbatch(off, ind, w.seeds.numpy(), so, w.cfg.fanout, rng_seed=1)
    assert not np.array_equal(other["ids"][:r["ids_offsets"][1]], r["ids"][:r["ids_offsets"][1]])
