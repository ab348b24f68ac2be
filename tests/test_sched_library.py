"""The library's frame scheduler against the scheduling oracle and the pool model, step by step,
on a host-only pool (no GPU): which streams are listed in which step, request ids, evictions,
and the block state that results from running the steps."""
import numpy as np
import pytest

from oracle import schedule as S
from oracle.pool_model import ACTION, DECODE, PoolModel
from paper_2603_14371_amd import binding as B


def _host_pool(num_blocks, free_order=None, **kw):
    cfg = B.make_config(2, num_blocks, free_order=free_order, flags=B.POOL_HOST_ONLY, **kw)
    return B.oxy_pool_create(cfg)


def _run(arrivals, k, s_act, chunk, mode, max_active, prefix_len=40, num_blocks=4096, seed=0):
    """Drives library scheduler + pool, and oracle schedule + pool model, through the same
    arrivals; compares every step; returns per-frame decode batch sizes."""
    rng = np.random.default_rng(seed)
    order = rng.permutation(num_blocks).astype(np.int32)
    pool = _host_pool(num_blocks, free_order=order, max_q_tokens=4096, max_append_tokens=4096)
    model = PoolModel(num_blocks, 16, 2, order.tolist())
    sched = B.oxy_sched_create(pool, k, s_act, chunk, max_active, mode)
    expect = S.simulate(arrivals, k, s_act, mode, max_active)
    sid_of_request, sizes = {}, []
    for t, targets in enumerate(arrivals):
        f = expect[t]
        act_sid, pids = [], []
        for n, want_rid in zip(targets, f["admitted"]):
            pid = B.oxy_prefix_create(pool)
            assert pid == model.prefix_create()
            for layer in range(2):
                B.oxy_prefix_append(pool, pid, layer, 0, 0, prefix_len, 0, 0)
                model.prefix_append(pid, layer, prefix_len, 0)
            rid = B.oxy_sched_admit(sched, pid, n)
            assert rid == want_rid
            # the library creates the action stream first, then the request's stream
            if s_act > 0:
                act_sid.append(model.stream_create(pid, ACTION))
            if rid >= 0:
                sid_of_request[rid] = model.stream_create(pid, DECODE)
                assert B.oxy_sched_request_info(sched, rid) == (sid_of_request[rid], 0, n, t)
            pids.append(pid)
        frame_sizes = []
        for act, dec in f["steps"]:
            items, n_action = B.oxy_sched_next_step(sched)
            want = [(act_sid[p], chunk) for p in act] + [(sid_of_request[r], 1) for r in dec]
            assert items == want and n_action == len(act)
            batch = B.oxy_batch_build(pool, items, B.BATCH_APPEND_ONLY, 0)
            slots = B.oxy_batch_slots(batch)
            B.oxy_batch_destroy(batch)
            assert slots == model.batch_build(items)
            if dec:
                frame_sizes.append(len(dec))
        assert B.oxy_sched_next_step(sched) == ([], 0)
        assert B.oxy_sched_next_step(sched) == ([], 0)        # asking again changes nothing
        with pytest.raises(B.OxyError):                       # no admission once steps were run
            if f["steps"]:
                B.oxy_sched_admit(sched, 0, 5)
            else:
                raise B.OxyError(-1, "frame without steps")
        assert B.oxy_sched_end_frame(sched) == f["finished"]
        for sid in act_sid:
            model.stream_release(sid)
        for rid in f["finished"]:
            model.stream_release(sid_of_request[rid])
        for pid in pids:
            model.prefix_release(pid)
        assert B.oxy_block_refcounts(pool, num_blocks) == model.ref
        assert B.oxy_free_blocks(pool) == model.free[::-1]
        sizes.append(frame_sizes)
        frame, n_active, n_created, n_rejected = B.oxy_sched_info(sched)
        assert frame == t + 1 and n_active == len(model.streams)
        assert n_rejected == sum(x.count(-1) for x in (g["admitted"] for g in expect[:t + 1]))
    B.oxy_sched_destroy(sched)
    assert B.oxy_pool_stats(pool) == (num_blocks, 0, 0)       # destroy released what was left
    B.oxy_pool_destroy(pool)
    return sizes


def test_worked_example_n12_k4():
    sizes = _run([[12]] * 9, k=4, s_act=2, chunk=5, mode=B.SCHED_BATCHED, max_active=0)
    assert sizes[0] == [1] * 4 and sizes[1] == [2] * 4 and all(s == [3] * 4 for s in sizes[2:])


@pytest.mark.parametrize("mode", [B.SCHED_BATCHED, B.SCHED_UNBATCHED, B.SCHED_UPPER_BOUND])
@pytest.mark.parametrize("pattern", ["uniform2", "poisson", "bursty_with_cap", "no_action"])
def test_random_arrivals_match_the_oracle(mode, pattern):
    rng = np.random.default_rng(100 * mode + len(pattern))
    s_act, chunk, max_active = 3, 7, 0
    if pattern == "uniform2":
        arrivals = [[int(rng.integers(1, 30)) for _ in range(2)] for _ in range(25)]
    elif pattern == "poisson":
        arrivals = [[int(rng.choice([4, 33])) for _ in range(rng.poisson(0.8))] for _ in range(40)]
    elif pattern == "bursty_with_cap":
        arrivals = [[int(rng.integers(5, 60)) for _ in range(int(rng.integers(0, 4)))]
                    for _ in range(30)]
        max_active = 5
    else:
        arrivals = [[int(rng.integers(1, 20))] for _ in range(20)]
        s_act, chunk = 0, 0
    arrivals += [[]] * 12
    _run(arrivals, k=6, s_act=s_act, chunk=chunk, mode=mode, max_active=max_active)


def test_scheduler_argument_errors():
    pool = _host_pool(64)
    for bad in (dict(k=0, denoise_steps=1, chunk=1), dict(k=1, denoise_steps=1, chunk=0),
                dict(k=1, denoise_steps=0, chunk=3), dict(k=1, denoise_steps=1, chunk=1, mode=7),
                dict(k=1, denoise_steps=1, chunk=1, max_active=-1)):
        with pytest.raises(B.OxyError) as e:
            B.oxy_sched_create(pool, **bad)
        assert e.value.code == B.ERR_INVALID_ARG
    sched = B.oxy_sched_create(pool, 4, 2, 3)
    with pytest.raises(B.OxyError) as e:
        B.oxy_sched_admit(sched, 99, 5)                       # no such prefix
    assert e.value.code == B.ERR_BAD_ID
    pid = B.oxy_prefix_create(pool)
    B.oxy_prefix_append(pool, pid, 0, 0, 0, 16, 0, 0)
    with pytest.raises(B.OxyError):
        B.oxy_sched_admit(sched, pid, 0)                      # empty request
    assert B.oxy_pool_stats(pool)[2] == 0                     # failed admissions left no stream
    assert B.oxy_sched_admit(sched, pid, 5) == 0
    with pytest.raises(B.OxyError):
        B.oxy_sched_admit(sched, pid, 5)                      # same observation twice
    with pytest.raises(B.OxyError):
        B.oxy_sched_end_frame(sched)                          # steps still to run
    with pytest.raises(B.OxyError) as e:
        B.oxy_sched_request_info(sched, 3)
    assert e.value.code == B.ERR_BAD_ID
    B.oxy_sched_destroy(sched)
    assert B.oxy_pool_stats(pool) == (64, 0, 0)
    B.oxy_pool_destroy(pool)


def test_calibrated_budget_matches_the_oracle():
    """The library's closed form of the steady-state frame against the oracle's simulation."""
    from oracle import schedule as S
    rng = np.random.default_rng(3)
    for _ in range(40):
        n, r, s_act = int(rng.integers(1, 40)), int(rng.integers(1, 4)), int(rng.integers(0, 8))
        size = r * n + 1
        t_mixed = np.sort(rng.uniform(50, 400, size)).tolist()
        t_dec = np.sort(rng.uniform(10, 200, size)).tolist()
        t_obs = float(rng.uniform(0, 300))
        budget = float(rng.uniform(200, 6000))
        want = S.calibrate_k(s_act, n, r, t_obs, t_mixed, t_dec, 1.0 / budget)
        got = B.oxy_sched_calibrate(t_mixed, t_dec, t_obs, s_act, n, r, budget)
        assert got[0] == want[0] and abs(got[1] - want[1]) <= 1e-9 * max(1.0, want[1])
    with pytest.raises(B.OxyError):       # batch sizes beyond the measured tables
        B.oxy_sched_calibrate([1.0, 2.0], [1.0, 2.0], 0.0, 2, 12, 1, 100.0)
    with pytest.raises(B.OxyError):
        B.oxy_sched_calibrate([1.0], [1.0], 0.0, 2, 0, 1, 100.0)
