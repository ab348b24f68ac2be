"""Pins of the scheduling oracle (oracle/schedule.py): the paper's worked example, the
B = N / k rule, token conservation, Little's law under random arrivals, and the ablation
variants.  No GPU."""
import math
import os

import numpy as np
import pytest

from oracle import schedule as S

GOLDEN = os.path.join(os.path.dirname(__file__), "golden")


def _fig3():
    vals = {}
    for line in open(os.path.join(GOLDEN, "schedule_fig3.txt")):
        if not line.startswith("#") and line.strip():
            key, v = line.split()
            vals[key] = int(v)
    return vals


def test_worked_example_of_the_timeline_figure():
    """Fig. 3: N = 12, k = 4, one observation per frame -> after warm-up three requests advance
    four tokens each per frame; request ids equal frame indices (App. A.2)."""
    g = _fig3()
    frames = S.simulate([[g["N"]]] * 10, k=g["k"], denoise_steps=2)
    sizes = S.decode_batch_sizes(frames)
    assert sizes[0] == [1] * g["k"] and sizes[1] == [2] * g["k"]
    for t in range(g["N"] // g["k"] - 1, 10):
        assert sizes[t] == [g["B"]] * g["k"]
    assert [f["admitted"] for f in frames] == [[t] for t in range(10)]
    # the request born in frame t leaves at the end of frame t + N/k - 1
    assert [f["finished"] for f in frames] == [[], []] + [[t] for t in range(8)]


@pytest.mark.parametrize("r,n,k", [(1, 12, 4), (2, 20, 5), (3, 64, 8), (4, 10, 10)])
def test_steady_state_batch_is_r_n_over_k(r, n, k):
    """Sec. 4.2: B = N / k for one arrival per frame; r arrivals per frame scale it by r."""
    frames = S.simulate([[n] * r] * 40, k=k, denoise_steps=3)
    for sizes in S.decode_batch_sizes(frames)[n // k:]:
        assert sizes == [r * n // k] * k


def test_every_request_gets_its_tokens_at_most_k_per_frame():
    rng = np.random.default_rng(5)
    arrivals = [[int(x) for x in rng.integers(1, 70, size=rng.poisson(1.3))] for _ in range(300)]
    arrivals += [[] for _ in range(40)]                       # drain
    k, s_act = 7, 4
    frames = S.simulate(arrivals, k=k, denoise_steps=s_act)
    target, birth, got, last = {}, {}, {}, {}
    for t, f in enumerate(frames):
        for rid, n in zip(f["admitted"], arrivals[t]):
            target[rid], birth[rid], got[rid] = n, t, 0
        assert sorted(f["admitted"]) == f["admitted"]
        per_frame = {}
        seen_empty = set()
        for act, dec in f["steps"]:
            assert len(set(dec)) == len(dec) and dec == sorted(dec)
            for rid in dec:
                assert rid not in seen_empty          # a request's tokens are consecutive steps
                per_frame[rid] = per_frame.get(rid, 0) + 1
            seen_empty |= set(per_frame) - set(dec)
        for rid, c in per_frame.items():
            assert c <= k
            got[rid] += c
            last[rid] = t
        # steps of the frame: the chunk needs s_act steps when something arrived
        n_act = sum(1 for act, _ in f["steps"] if act)
        assert n_act == (s_act if arrivals[t] else 0)
        for rid in f["finished"]:
            assert got[rid] == target[rid] and last[rid] == t
    assert got == target
    assert list(target) == list(range(len(target)))           # sequential ids, none reused
    for rid in target:                                        # lifetime = ceil(N / k) frames
        assert last[rid] - birth[rid] + 1 == math.ceil(target[rid] / k)


def test_littles_law_under_poisson_arrivals():
    """Mean number of requests decoding per frame = arrival rate x mean lifetime in frames."""
    rng = np.random.default_rng(11)
    lam, k = 1.5, 8
    arrivals = [[int(rng.choice([16, 64])) for _ in range(rng.poisson(lam))] for _ in range(6000)]
    frames = S.simulate(arrivals, k=k, denoise_steps=2)
    in_flight = [max(sz) if sz else 0 for sz in S.decode_batch_sizes(frames)]
    expect = lam * (0.5 * 2 + 0.5 * 8)
    assert abs(np.mean(in_flight[100:]) - expect) < 0.06 * expect


def test_unbatched_variant_serves_one_request_at_a_time_to_completion():
    arrivals = [[5, 9], [3], [], [20]]
    frames = S.simulate(arrivals, k=4, denoise_steps=6, mode=S.UNBATCHED)
    for f, targets in zip(frames, arrivals):
        assert all(len(dec) <= 1 and len(act) <= 1 for act, dec in f["steps"])
        assert len(f["steps"]) == sum(max(6, n) for n in targets)
        assert f["finished"] == f["admitted"]
    first = frames[0]["steps"]
    assert first[0] == ([0], [0]) and first[4] == ([0], [0]) and first[5] == ([0], [])
    assert first[6] == ([1], [1]) and first[14] == ([], [1])


def test_upper_bound_variant_drops_the_rest_of_each_request():
    arrivals = [[30], [30, 2], [30]]
    frames = S.simulate(arrivals, k=4, denoise_steps=3, mode=S.UPPER_BOUND)
    assert S.decode_batch_sizes(frames) == [[1] * 4, [2, 2, 1, 1], [1] * 4]
    assert [f["finished"] for f in frames] == [[0], [1, 2], [3]]


def test_full_active_set_serves_the_action_only():
    frames = S.simulate([[40]] * 8, k=4, denoise_steps=2, max_active=3)
    assert [f["admitted"] for f in frames[:5]] == [[0], [1], [2], [-1], [-1]]
    assert all(len(dec) <= 3 for f in frames for _, dec in f["steps"])
    assert all(sum(1 for act, _ in f["steps"] if act) == 2 for f in frames)


def test_steady_frame_time_of_the_worked_example_by_hand():
    """Fig. 3 shape (N = 12, k = 4, one arrival per frame) with S = 2: the steady frame has two
    mixed steps and two decode-only steps, each with three requests decoding."""
    t_mixed = [10.0, 11.0, 12.0, 13.0, 14.0]
    t_dec = [0.0, 3.0, 3.5, 4.0, 4.5]
    t = S.steady_frame_time(4, 2, 12, 1, t_obs=20.0, t_mixed=t_mixed, t_decode=t_dec)
    assert t == 20.0 + 2 * 13.0 + 2 * 4.0
    # N not a multiple of k: N = 10, k = 4 -> ages 0, 1 decode 4 tokens, age 2 decodes 2
    t = S.steady_frame_time(4, 2, 10, 1, 20.0, t_mixed, t_dec)
    assert t == 20.0 + 2 * 13.0 + 2 * 3.5
    # budget below S: the denoise steps beyond k carry no decoding
    t = S.steady_frame_time(1, 3, 3, 1, 20.0, t_mixed, t_dec)
    assert t == 20.0 + 13.0 + 2 * 10.0


def test_calibrated_budget_is_the_largest_that_meets_the_rate():
    n = 24
    t_mixed = [100.0 + 2.0 * b for b in range(2 * n + 1)]
    t_dec = [40.0 + 2.0 * b for b in range(2 * n + 1)]
    # closed form for k | N, one arrival per frame, k >= S: T = t_obs + S t_mixed[N/k] + (k-S) t_dec[N/k]
    s_act, t_obs = 4, 200.0
    for k in (4, 6, 8, 12, 24):
        b = n // k
        want = t_obs + s_act * t_mixed[b] + (k - s_act) * t_dec[b]
        assert S.steady_frame_time(k, s_act, n, 1, t_obs, t_mixed, t_dec) == want
    budget_us = 1000.0
    k, t = S.calibrate_k(s_act, n, 1, t_obs, t_mixed, t_dec, 1.0 / budget_us)
    assert 1 <= k < n and t <= budget_us
    for bigger in range(k + 1, n + 1):
        assert S.steady_frame_time(bigger, s_act, n, 1, t_obs, t_mixed, t_dec) > budget_us
    assert S.calibrate_k(s_act, n, 1, t_obs, t_mixed, t_dec, 1.0 / 100.0) == (0, 0.0)
    assert S.calibrate_k(s_act, n, 1, t_obs, t_mixed, t_dec, 1.0 / 1e9)[0] == n
