"""Scheduling oracle: the per-frame execution flow of the paper as a plain simulation.

Test infrastructure only; shares no code with the C++ frame scheduler it checks.

The paper's Alg. 1 (App. A.3; Sec. 3.2, "Per-frame execution flow") handles one new
observation per frame: prefill, action denoising over S steps, a fresh language
request stored under the next request id (App. A.2: the id is the number of requests
created so far), then every active request advances by the per-frame budget k, and
finished requests are evicted while the rest persist.  Sec. 4.4 generalises the
arrivals (several or no observations per frame, random lengths) and Sec. 4.3 names
the ablation variants.  This module writes that flow out for an arbitrary arrival
sequence, one decision at a time, with nothing precomputed:

* frame t admits its arrivals in order; each gets an action chunk (denoised over S
  steps) and, while the active set has room, a language request with a target
  length N (termination by length only: there are no logits, hence no EOS);
* step s of a frame lists the chunk of every observation admitted in this frame
  while s < S, and one token for every active request that has not finished and
  has used fewer than k steps of this frame's budget; a frame has as many steps as
  the longest of these needs (readings: the mixed step carries denoise step s and
  decode token s together; a finished request stops being listed at once);
* at frame end the finished requests leave the active set, in id order.

Variants (Sec. 4.3): "batched" is the flow above; "unbatched" is cross-task sharing
without cross-frame batching: each observation is served alone and its request runs
to completion before the next one starts, so nothing carries over; "upper_bound" is
the single-frame decoding oracle of the ablation: k tokens are decoded and the rest
of the request is dropped at frame end.

Budget calibration (Sec. 3.2: k is chosen offline from the target frame rate and the hardware
so that batched decoding over the typical active batch fits into what remains of the frame
after action denoising): `steady_frame_time` prices the steps of a steady-state frame, found
by running the simulation until it is periodic, with measured per-step costs; `calibrate_k`
is the definition itself, the largest k whose steady-state frame still meets the rate.

What pins it (tests/test_oracle_schedule.py): the worked example of Fig. 3 (N = 12,
k = 4 -> three requests in parallel, four tokens each per frame), the rule B = N / k
of Sec. 4.2 and its extension r N / k for r arrivals per frame, token conservation
(every request receives exactly N tokens, at most k per frame), and Little's law for
random arrivals.
"""

BATCHED = 0
UNBATCHED = 1
UPPER_BOUND = 2


class Request:
    def __init__(self, rid, frame, target):
        self.rid = rid
        self.birth = frame
        self.target = target
        self.done = 0


def simulate(arrivals, k, denoise_steps, mode=BATCHED, max_active=0):
    """arrivals[t] = list of target lengths N of the observations that arrive in frame t
    (an empty list: no observation in that frame).  Returns a list of frames; a frame is
    a dict with
      steps:    list of steps, a step = (action, decode) with action = positions (within
                this frame's arrivals) of the observations whose chunk is denoised in this
                step and decode = ids of the requests that decode one token in it;
      admitted: request id per arrival, or -1 when the active set was full;
      finished: ids evicted at the end of the frame (ascending)."""
    active = []          # requests in id order
    n_created = 0
    frames = []
    for t, targets in enumerate(arrivals):
        admitted = []
        fresh = []
        for target in targets:
            if target < 1:
                raise ValueError("target length must be positive")
            if max_active and len(active) >= max_active:
                admitted.append(-1)
                continue
            r = Request(n_created, t, target)
            n_created += 1
            active.append(r)
            fresh.append(r)
            admitted.append(r.rid)
        steps = []
        if mode == UNBATCHED:
            # one observation at a time, its request alone and to completion
            for pos, rid in enumerate(admitted):
                r = next((x for x in fresh if x.rid == rid), None)
                s = 0
                while s < denoise_steps or (r is not None and r.done < r.target):
                    act = [pos] if s < denoise_steps else []
                    dec = []
                    if r is not None and r.done < r.target:
                        dec.append(r.rid)
                        r.done += 1
                    steps.append((act, dec))
                    s += 1
        else:
            s = 0
            while True:
                act = list(range(len(targets))) if s < denoise_steps else []
                dec = []
                if s < k:
                    for r in active:
                        if r.done < r.target:
                            dec.append(r.rid)
                            r.done += 1
                if not act and not dec:
                    break
                steps.append((act, dec))
                s += 1
        if mode == UPPER_BOUND:
            finished = [r.rid for r in active]
        else:
            finished = [r.rid for r in active if r.done >= r.target]
        active = [r for r in active if r.rid not in finished]
        frames.append({"steps": steps, "admitted": admitted, "finished": finished})
    return frames


def decode_batch_sizes(frames):
    """Number of requests decoding in each step that decodes at all, per frame."""
    return [[len(dec) for _, dec in f["steps"] if dec] for f in frames]


def steady_frame_time(k, denoise_steps, target, arrivals_per_frame, t_obs, t_mixed, t_decode):
    """Time of one frame once the schedule has become periodic: every arriving observation
    costs t_obs (its prefill stand-in and fan-out), a step that denoises costs t_mixed[b] and a
    decode-only step t_decode[b], b = number of requests decoding in that step."""
    lifetime = -(-target // k)
    frames = simulate([[target] * arrivals_per_frame] * (lifetime + 2), k, denoise_steps)
    total = arrivals_per_frame * t_obs
    for act, dec in frames[-1]["steps"]:
        total += t_mixed[len(dec)] if act else t_decode[len(dec)]
    return total


def calibrate_k(denoise_steps, target, arrivals_per_frame, t_obs, t_mixed, t_decode, target_hz):
    """Largest per-frame budget k in 1..target whose steady-state frame time stays within
    1 / target_hz; 0 if there is none.  Returns (k, frame time at that k)."""
    best = (0, 0.0)
    for k in range(1, target + 1):
        t = steady_frame_time(k, denoise_steps, target, arrivals_per_frame, t_obs, t_mixed,
                              t_decode)
        if t <= 1.0 / target_hz:
            best = (k, t)
    return best
