"""The rule the GPU path uses to find every iteration's threshold bucket before the loop runs
(Section 3.4's recurrence): the candidates per next-use bucket are the
residents the iteration does not access plus the iteration's accesses by their new key, the
number to drop is the candidates beyond the capacity, and the residents' histogram rolls
forward by the rule itself.  Checked here on the CPU against the sort-based definition of the
recurrence (keep the `cap` smallest (next accessed iteration, id) of cache ∪ accesses), with
no code shared with the kernels or the oracle."""
import numpy as np


def next_use(tr, S):
    last, nxt = {}, [None] * S
    for i in range(S - 1, -1, -1):
        nxt[i] = np.array([last.get(int(v), S) for v in tr[i]], dtype=np.int64)
        for v in tr[i]:
            last[int(v)] = i
    return nxt, dict(last)


def test_threshold_bucket_and_dropped_count_follow_from_histograms_alone():
    rng = np.random.default_rng(5)
    for trial in range(300):
        n = int(rng.integers(2, 300))
        S = int(rng.integers(1, 14))
        cap = int(rng.integers(1, n + 1))
        tr = [rng.choice(n, size=rng.integers(0, min(int(rng.integers(1, 150)), n) + 1), replace=False)
              for _ in range(S)]
        nxt, first = next_use(tr, S)
        res = dict(sorted(first.items(), key=lambda kv: (kv[1], kv[0]))[:cap])   # C_0: row -> key
        R = np.zeros(S + 1, dtype=np.int64)
        for f in res.values():
            R[f] += 1
        for i in range(S):
            # the definition, on the state
            cand = dict(res)
            for v, k in zip(tr[i], nxt[i]):
                cand[int(v)] = int(k)
            items = sorted(cand.items(), key=lambda kv: (kv[1], kv[0]))
            kept, dropped = items[:cap], items[cap:]
            # the rule, on histograms
            C = R.copy()
            C[i] = 0                                     # the residents keyed to i are accessed
            C += np.bincount(nxt[i], minlength=S + 1)
            assert C.sum() == len(cand)
            drop = max(0, int(C.sum()) - cap)
            assert drop == len(dropped)
            jstar, rem, cum = S + 1, 0, 0
            for j in range(S, -1, -1):                   # from "never" downwards
                if drop > 0 and cum <= drop < cum + C[j]:
                    jstar, rem = j, drop - cum
                    break
                cum += C[j]
            if dropped:
                lowest = min(k for _, k in dropped)
                gone = sum(1 for _, k in dropped if k == lowest)
                if gone < C[lowest]:                     # the bucket is cut
                    assert (lowest, gone) == (jstar, rem), (trial, i)
                else:                                    # it goes whole: the walk stops below it, nothing to cut
                    assert jstar < lowest and rem == 0, (trial, i)
            # the residents of the next iteration by key, both ways
            res = dict(kept)
            want = np.zeros(S + 1, dtype=np.int64)
            for k in res.values():
                want[k] += 1
            roll = np.array([C[j] if j < jstar else C[j] - rem if j == jstar else 0
                             for j in range(S + 1)])
            assert np.array_equal(roll, want), (trial, i)
            R = roll
