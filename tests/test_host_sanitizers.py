"""The host side of the library (block pool, batch builder, scheduler) compiled with gcc under
AddressSanitizer + UndefinedBehaviorSanitizer, with CPU stand-ins for the HIP runtime and the
kernel launchers (tests/hostbuild), replaying random operation sequences whose every status,
id, slot list and pool state is written down beforehand from the pool model.  The pool is a
full one ("device" buffers are host memory of exactly the advertised size), so the descriptor
upload of every batch runs under the sanitizer too.  Also forces device failures from the host
and checks that a failing call leaves the pool untouched.  No GPU."""
import os
import shutil
import subprocess

import numpy as np
import pytest

from oracle.pool_model import PoolError, PoolModel

ROOT = os.path.dirname(os.path.dirname(os.path.abspath(__file__)))
HB = os.path.join(ROOT, "tests", "hostbuild")
CSRC = os.path.join(ROOT, "paper_2603_14371_amd", "csrc")
ERR_DEVICE = -7


@pytest.fixture(scope="module")
def replay_exe(tmp_path_factory):
    gxx = shutil.which("g++")
    if gxx is None:
        pytest.skip("no g++")
    exe = str(tmp_path_factory.mktemp("hostbuild") / "replay_asan")
    cmd = [gxx, "-std=c++17", "-O1", "-g", "-fsanitize=address,undefined",
           "-fno-sanitize-recover=undefined", "-fno-omit-frame-pointer", "-w",
           "-D__HIP_PLATFORM_AMD__", "-I/opt/rocm/include",
           os.path.join(CSRC, "oxy_pool.cpp"), os.path.join(CSRC, "oxy_sched.cpp"),
           os.path.join(HB, "hip_stubs.cpp"), os.path.join(HB, "replay_main.cpp"), "-o", exe]
    res = subprocess.run(cmd, stdout=subprocess.PIPE, stderr=subprocess.STDOUT, text=True)
    assert res.returncode == 0, res.stdout[-3000:]
    return exe


def _run(exe, tmp_path, script):
    path = tmp_path / "script.txt"
    path.write_text("\n".join(" ".join(str(int(x)) for x in line) for line in script) + "\n")
    env = dict(os.environ, ASAN_OPTIONS="detect_leaks=1:abort_on_error=0", UBSAN_OPTIONS="print_stacktrace=1")
    res = subprocess.run([exe, str(path)], stdout=subprocess.PIPE, stderr=subprocess.STDOUT,
                         text=True, env=env, timeout=300)
    assert res.returncode == 0 and res.stdout.startswith("OK"), res.stdout[-4000:]
    return res.stdout


def _state(model):
    line = [10, model.num_blocks] + list(model.ref) + [len(model.free)] + model.free[::-1]
    line.append(len(model.streams))
    for sid, s in model.streams.items():
        line += [sid, s.prefix_id, s.kind, s.length, len(s.blocks)] + list(s.blocks)
    line.append(len(model.prefixes))
    for pid, p in model.prefixes.items():
        line += [pid, p.length, len(p.blocks), int(p.sealed), p.n_streams] + list(p.blocks)
    return line


def _try(fn):
    try:
        return 0, fn()
    except PoolError as e:
        return e.code, None


def _fuzz_script(seed, n_ops, nb=200, inject=False):
    rng = np.random.default_rng(seed)
    order = rng.permutation(nb).tolist()
    model = PoolModel(nb, 16, 2, order)
    script = [[0, nb, 2, 1, 256, nb] + order]
    prefixes = []
    n_injected = 0
    for _ in range(n_ops):
        r = rng.random()
        fail_now = inject and rng.random() < 0.25
        if r < 0.1:
            pid = model.prefix_create()
            prefixes.append(pid)
            script.append([1, pid])
        elif r < 0.14 and prefixes:
            parent = int(rng.choice(prefixes + [98]))
            plen = model.prefixes[parent].length if parent in model.prefixes else 0
            n = int(rng.choice([0, 16 * int(rng.integers(0, plen // 16 + 1)), plen, plen + 16, 8]))
            st, pid = _try(lambda: model.prefix_fork(parent, n))
            if st == 0:
                prefixes.append(pid)
            script.append([3, parent, n, st, -1 if pid is None else pid])
        elif r < 0.27 and prefixes:
            pid = int(rng.choice(prefixes + [99]))
            n, layer = int(rng.integers(0, 70)), int(rng.integers(0, 3))
            plen = model.prefixes[pid].length if pid in model.prefixes else 0
            frozen = model.prefixes[pid].frozen if pid in model.prefixes else 0
            pos0 = int(rng.choice([0, plen, plen + 1, frozen, max(0, plen - 5)]))
            if fail_now:     # would the call reach its launch?  then the launch fails
                probe = PoolModel.__new__(PoolModel)
                probe.__dict__ = _clone(model)
                st, _ = _try(lambda: probe.prefix_append(pid, layer, n, pos0))
                if st == 0:
                    script.append([9, 0, 1])
                    script.append([2, pid, layer, n, pos0, ERR_DEVICE])
                    n_injected += 1
                    script.append(_state(model))
                    continue
            st, _ = _try(lambda: model.prefix_append(pid, layer, n, pos0))
            script.append([2, pid, layer, n, pos0, st])
        elif r < 0.4:
            pid = int(rng.choice(prefixes + [-1, 77])) if prefixes else -1
            kind = int(rng.integers(0, 3))
            st, sid = _try(lambda: model.stream_create(pid, kind))
            script.append([5, pid, kind, st, -1 if sid is None else sid])
        elif r < 0.75 and model.streams:
            ids = list(model.streams) + ([12345] if rng.random() < 0.05 else [])
            sids = rng.permutation(ids)[:int(rng.integers(1, 6))]
            lo = 0 if rng.random() < 0.05 else 1
            items = [(int(s), int(rng.integers(lo, 40))) for s in sids]
            if rng.random() < 0.05:
                items.append(items[0])
            flags = int(rng.random() < 0.2)
            flat = [x for it in items for x in it]
            if fail_now:
                probe = PoolModel.__new__(PoolModel)
                probe.__dict__ = _clone(model)
                st, _ = _try(lambda: probe.batch_build(items))
                if st == 0:
                    script.append([9, int(rng.integers(0, 2)), 1])   # the copy, or its event
                    script.append([8, flags, len(items)] + flat + [ERR_DEVICE, 0])
                    script.append([9, 0, 0])
                    n_injected += 1
                    script.append(_state(model))
                    continue
            st, slots = _try(lambda: model.batch_build(items))
            slots = slots or []
            script.append([8, flags, len(items)] + flat + [st, len(slots)] + slots)
        elif r < 0.87 and model.streams:
            sid = int(rng.choice(list(model.streams) + [4242]))
            st, _ = _try(lambda: model.stream_release(sid))
            script.append([6, sid, st])
        elif r < 0.93 and prefixes:
            pid = int(rng.choice(prefixes))
            st, _ = _try(lambda: model.prefix_release(pid))
            script.append([4, pid, st])
        elif model.streams:
            sid = int(rng.choice(list(model.streams)))
            new_len = int(rng.integers(0, model.streams[sid].length + 2))
            st, _ = _try(lambda: model.stream_rewind(sid, new_len))
            script.append([7, sid, new_len, st])
        script.append(_state(model))
    return script, n_injected


def _clone(model):
    import copy
    return copy.deepcopy(model.__dict__)


@pytest.mark.parametrize("seed", range(3))
def test_random_sequences_under_asan_ubsan(replay_exe, tmp_path, seed):
    script, _ = _fuzz_script(2000 + seed, 700)
    out = _run(replay_exe, tmp_path, script)
    assert int(out.split()[1]) == len(script)


def test_device_failures_leave_the_pool_unchanged(replay_exe, tmp_path):
    """A HIP call that fails inside oxy_prefix_append (the launch) or oxy_batch_build (the
    descriptor copy or its event) gives OXY_ERR_DEVICE and changes no block, refcount, length or
    free-stack position."""
    script, n = _fuzz_script(3001, 900, inject=True)
    assert n > 25
    _run(replay_exe, tmp_path, script)
