"""Pins for the oracle's regeneration-loop reductions (Section 3.4: samples are
tried until one verifies or the attempts run out; Section 4.2: Pass@K, average
and maximum number of attempts).  None of the expected values comes from the
functions under test: closed forms, hand-written cases and a plain Python loop."""
import numpy as np

from oracle import vlo


def verdicts(statuses):
    r = np.zeros(len(statuses), vlo.RESULT_DTYPE)
    r["status"] = statuses
    r["where"] = np.arange(len(statuses)) * 7 + 1   # the reductions must not look at these
    return r


def test_hand_written_cases():
    s = vlo.summarize(verdicts([3, 1, 0, 2, 0]))[0]
    assert (s["first_ok"], s["passed"], list(s["hist"])) == (2, 1, [2, 1, 1, 1])
    s = vlo.summarize(verdicts([0]))[0]
    assert (s["first_ok"], s["passed"], list(s["hist"])) == (0, 1, [1, 0, 0, 0])
    # every attempt fails: the loop is exhausted, first_ok = K
    s = vlo.summarize(verdicts([3, 3, 2, 1]))[0]
    assert (s["first_ok"], s["passed"], list(s["hist"])) == (4, 0, [0, 1, 1, 2])


def test_closed_forms():
    for K in (1, 7, 100, 1000):
        ok = vlo.summarize(verdicts(np.zeros(K, np.uint32)))[0]
        assert ok["first_ok"] == 0 and ok["passed"] == 1 and list(ok["hist"]) == [K, 0, 0, 0]
        bad = vlo.summarize(verdicts(np.full(K, 3, np.uint32)))[0]
        assert bad["first_ok"] == K and bad["passed"] == 0 and list(bad["hist"]) == [0, 0, 0, K]
        for j in (0, K // 2, K - 1):   # a single accepted sample at position j
            st = np.full(K, 1, np.uint32)
            st[j] = 0
            one = vlo.summarize(verdicts(st))[0]
            assert one["first_ok"] == j and one["passed"] == 1 and one["hist"].sum() == K


def test_against_a_python_loop():
    rng = np.random.default_rng(5)
    sums, Ks, tries = [], [], []
    for _ in range(200):
        K = int(rng.integers(1, 130))
        st = rng.choice(4, K, p=[0.1, 0.3, 0.3, 0.3]).astype(np.uint32)
        s = vlo.summarize(verdicts(st))[0]
        first = K
        for k in range(K):          # the loop of Section 3.4: stop at the first accepted sample
            if st[k] == 0:
                first = k
                break
        assert s["first_ok"] == first and s["passed"] == int(first < K)
        assert list(s["hist"]) == [int((st == x).sum()) for x in range(4)]
        sums.append(s)
        Ks.append(K)
        tries.append(first + 1 if first < K else K)
    loop = vlo.loop_stats(np.array(sums, vlo.SUMMARY_DTYPE), Ks)[0]
    assert loop["n_passed"] == sum(int(s["passed"]) for s in sums)
    assert loop["max_tries"] == max(tries) and loop["sum_tries"] == sum(tries)
    assert list(loop["hist"]) == [sum(int(s["hist"][x]) for s in sums) for x in range(4)]


def test_attempt_counts_of_a_passing_suite():
    """Every kernel passes at its first sample: one attempt each (the best case the
    paper's AvgTry / MaxTry can take)."""
    sums = np.array([vlo.summarize(verdicts([0, 3, 3]))[0] for _ in range(10)], vlo.SUMMARY_DTYPE)
    loop = vlo.loop_stats(sums, [3] * 10)[0]
    assert loop["n_passed"] == 10 and loop["max_tries"] == 1 and loop["sum_tries"] == 10
    # and an exhausted kernel costs all its attempts
    sums[3] = vlo.summarize(verdicts([1, 2, 3]))[0]
    loop = vlo.loop_stats(sums, [3] * 10)[0]
    assert loop["n_passed"] == 9 and loop["max_tries"] == 3 and loop["sum_tries"] == 12
