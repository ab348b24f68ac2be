// Frame scheduler: the paper's per-frame execution flow (Alg. 1, App. A.3; Sec. 3.2) over the
// streams of one pool, generalised to any number of observations per frame (Sec. 4.4) and with
// the variants of the ablation (Sec. 4.3).  Host logic only: it decides which streams are
// listed in which step; the caller runs the steps (oxy_batch_build + attention).  It talks to
// the pool through the public calls of oxy.h.
#include "../../include/oxy.h"

#include <algorithm>
#include <cstdarg>
#include <cstdio>
#include <new>
#include <vector>

extern "C" __attribute__((visibility("hidden"))) void oxy_internal_set_error(const char* msg);

namespace {

int32_t fail(int32_t code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof(buf), fmt, ap);
  va_end(ap);
  oxy_internal_set_error(buf);
  return code;
}

struct Request {        // the KV part of one language request state (Eq. 3)
  int32_t rid, sid, target, done, birth, used;   // used: tokens decoded in the current frame
};
struct Observation {    // one observation admitted in the current frame
  int32_t prefix_id, action_sid, rid;            // rid = -1: the active set was full
};

}  // namespace

struct oxy_sched {
  oxy_pool* pool = nullptr;
  oxy_sched_config cfg{};
  std::vector<Request> active;      // ascending request id
  std::vector<Observation> fresh;
  int32_t frame = 0, n_created = 0, n_rejected = 0;
  int32_t step = 0;                 // steps handed out in this frame
  int32_t cur_obs = 0, cur_step = 0;   // unbatched variant: observation being served, its step
};

namespace {

Request* find_request(oxy_sched* s, int32_t rid) {
  for (Request& r : s->active)
    if (r.rid == rid) return &r;
  return nullptr;
}

// Items of the next step without committing it.  Unbatched: advances the cursor past
// observations that need nothing more (that is not a visible state change).
void plan_step(oxy_sched* s, std::vector<oxy_item>& items, int32_t* n_action,
               std::vector<Request*>& decoding) {
  const oxy_sched_config& c = s->cfg;
  items.clear();
  decoding.clear();
  *n_action = 0;
  if (c.mode == OXY_SCHED_UNBATCHED) {
    while (s->cur_obs < (int32_t)s->fresh.size()) {
      const Observation& o = s->fresh[s->cur_obs];
      Request* r = o.rid >= 0 ? find_request(s, o.rid) : nullptr;
      if (o.action_sid >= 0 && s->cur_step < c.denoise_steps) {
        items.push_back({o.action_sid, c.chunk});
        *n_action = 1;
      }
      if (r && r->done < r->target) {
        items.push_back({r->sid, 1});
        decoding.push_back(r);
      }
      if (!items.empty()) return;
      s->cur_obs++;
      s->cur_step = 0;
    }
    return;
  }
  if (s->step < c.denoise_steps)
    for (const Observation& o : s->fresh)
      if (o.action_sid >= 0) {
        items.push_back({o.action_sid, c.chunk});
        ++*n_action;
      }
  if (s->step < c.k)
    for (Request& r : s->active)
      if (r.done < r.target) {
        items.push_back({r.sid, 1});
        decoding.push_back(&r);
      }
}

}  // namespace

extern "C" {

int32_t oxy_sched_create(oxy_pool* pool, const oxy_sched_config* cfg, oxy_sched** out) {
  if (!pool || !cfg || !out) return fail(OXY_ERR_INVALID_ARG, "sched_create: null argument");
  *out = nullptr;
  if (cfg->k < 1 || cfg->denoise_steps < 0 || cfg->chunk < 0 || cfg->max_active < 0 ||
      cfg->mode < OXY_SCHED_BATCHED || cfg->mode > OXY_SCHED_UPPER_BOUND ||
      (cfg->denoise_steps > 0) != (cfg->chunk > 0))
    return fail(OXY_ERR_INVALID_ARG, "sched_create: k %d, denoise_steps %d, chunk %d, max_active %d, mode %d",
                cfg->k, cfg->denoise_steps, cfg->chunk, cfg->max_active, cfg->mode);
  oxy_sched* s = new (std::nothrow) oxy_sched();
  if (!s) return fail(OXY_ERR_INVALID_ARG, "sched_create: out of host memory");
  s->pool = pool;
  s->cfg = *cfg;
  *out = s;
  return OXY_OK;
}

int32_t oxy_sched_destroy(oxy_sched* s) {
  if (!s) return fail(OXY_ERR_INVALID_ARG, "sched_destroy: null");
  for (const Observation& o : s->fresh)
    if (o.action_sid >= 0) (void)oxy_stream_release(s->pool, o.action_sid);
  for (const Request& r : s->active) (void)oxy_stream_release(s->pool, r.sid);
  for (const Observation& o : s->fresh) (void)oxy_prefix_release(s->pool, o.prefix_id);
  delete s;
  return OXY_OK;
}

int32_t oxy_sched_admit(oxy_sched* s, int32_t prefix_id, int32_t target_len, int32_t* request_id) {
  if (!s || !request_id) return fail(OXY_ERR_INVALID_ARG, "sched_admit: null argument");
  if (s->step != 0 || s->cur_obs != 0 || s->cur_step != 0)
    return fail(OXY_ERR_INVALID_ARG, "sched_admit: frame %d already has steps", s->frame);
  if (target_len < 1) return fail(OXY_ERR_INVALID_ARG, "sched_admit: target length %d", target_len);
  for (const Observation& o : s->fresh)
    if (o.prefix_id == prefix_id)
      return fail(OXY_ERR_INVALID_ARG, "sched_admit: prefix %d admitted twice", prefix_id);
  Observation o{prefix_id, -1, -1};
  int32_t rc = OXY_OK;
  if (s->cfg.denoise_steps > 0) {
    rc = oxy_stream_create(s->pool, prefix_id, OXY_KIND_ACTION, &o.action_sid);
    if (rc != OXY_OK) return rc;
  }
  const bool room = s->cfg.max_active == 0 || (int32_t)s->active.size() < s->cfg.max_active;
  if (room) {
    int32_t sid = -1;
    rc = oxy_stream_create(s->pool, prefix_id, OXY_KIND_DECODE, &sid);
    if (rc != OXY_OK) {   // leave nothing behind
      if (o.action_sid >= 0) (void)oxy_stream_release(s->pool, o.action_sid);
      return rc;
    }
    o.rid = s->n_created++;
    s->active.push_back({o.rid, sid, target_len, 0, s->frame, 0});
  } else {
    s->n_rejected++;
  }
  s->fresh.push_back(o);
  *request_id = o.rid;
  return OXY_OK;
}

int32_t oxy_sched_next_step(oxy_sched* s, oxy_item* items, int32_t cap, int32_t* n_items,
                            int32_t* n_action_items) {
  if (!s || !items || !n_items) return fail(OXY_ERR_INVALID_ARG, "sched_next_step: null argument");
  std::vector<oxy_item> plan;
  std::vector<Request*> decoding;
  int32_t n_action = 0;
  plan_step(s, plan, &n_action, decoding);
  if ((int32_t)plan.size() > cap)
    return fail(OXY_ERR_INVALID_ARG, "sched_next_step: %zu items > cap %d", plan.size(), cap);
  std::copy(plan.begin(), plan.end(), items);
  *n_items = (int32_t)plan.size();
  if (n_action_items) *n_action_items = n_action;
  if (plan.empty()) return OXY_OK;      // the frame has no more steps
  for (Request* r : decoding) {
    r->done++;
    r->used++;
  }
  if (s->cfg.mode == OXY_SCHED_UNBATCHED)
    s->cur_step++;
  else
    s->step++;
  return OXY_OK;
}

int32_t oxy_sched_end_frame(oxy_sched* s, int32_t* finished, int32_t cap, int32_t* n_finished) {
  if (!s || !n_finished || (cap > 0 && !finished))
    return fail(OXY_ERR_INVALID_ARG, "sched_end_frame: null argument");
  {
    std::vector<oxy_item> plan;
    std::vector<Request*> decoding;
    int32_t n_action = 0;
    plan_step(s, plan, &n_action, decoding);
    if (!plan.empty())
      return fail(OXY_ERR_INVALID_ARG, "sched_end_frame: frame %d still has steps", s->frame);
  }
  int32_t n_done = 0;
  for (const Request& r : s->active)
    if (s->cfg.mode == OXY_SCHED_UPPER_BOUND || r.done >= r.target) n_done++;
  if (n_done > cap) return fail(OXY_ERR_INVALID_ARG, "sched_end_frame: %d finished > cap %d", n_done, cap);
  // order of the releases: action streams, finished requests by id, then the creator's
  // reference of every prefix admitted in this frame
  for (const Observation& o : s->fresh)
    if (o.action_sid >= 0) (void)oxy_stream_release(s->pool, o.action_sid);
  std::vector<Request> keep;
  keep.reserve(s->active.size());
  int32_t n = 0;
  for (Request& r : s->active) {
    if (s->cfg.mode == OXY_SCHED_UPPER_BOUND || r.done >= r.target) {
      (void)oxy_stream_release(s->pool, r.sid);
      finished[n++] = r.rid;
    } else {
      r.used = 0;
      keep.push_back(r);
    }
  }
  for (const Observation& o : s->fresh) (void)oxy_prefix_release(s->pool, o.prefix_id);
  s->active.swap(keep);
  s->fresh.clear();
  s->frame++;
  s->step = s->cur_obs = s->cur_step = 0;
  *n_finished = n;
  return OXY_OK;
}

int32_t oxy_sched_calibrate(const double* t_mixed, const double* t_decode, int32_t n_table,
                            double t_observation, int32_t denoise_steps, int32_t target_len,
                            int32_t arrivals_per_frame, double frame_budget, int32_t* k_out,
                            double* frame_time_out) {
  if (!t_mixed || !t_decode || !k_out || n_table < 1 || denoise_steps < 0 || target_len < 1 ||
      arrivals_per_frame < 1 || !(frame_budget > 0.0))
    return fail(OXY_ERR_INVALID_ARG, "sched_calibrate: null or non-positive argument");
  // Steady state under budget k with r arrivals per frame: a request lives ceil(N/k) frames, so
  // at step s of a frame r * (floor(N/k) + [s < N mod k]) requests decode (s < k), and the
  // frame has max(S, steps that decode) steps.
  int32_t best_k = 0;
  double best_t = 0.0;
  for (int32_t k = 1; k <= target_len; ++k) {
    const int32_t full = target_len / k, rem = target_len % k;
    const int32_t n_dec_steps = full > 0 ? k : rem;
    const int32_t n_steps = std::max(denoise_steps, n_dec_steps);
    double t = arrivals_per_frame * t_observation;
    for (int32_t s = 0; s < n_steps; ++s) {
      const int64_t b = s < n_dec_steps ? (int64_t)arrivals_per_frame * (full + (s < rem ? 1 : 0)) : 0;
      if (b >= n_table)
        return fail(OXY_ERR_INVALID_ARG, "sched_calibrate: batch %lld at k = %d is beyond the cost tables (%d)",
                    (long long)b, k, n_table);
      t += s < denoise_steps ? t_mixed[b] : t_decode[b];
    }
    if (t <= frame_budget) {
      best_k = k;
      best_t = t;
    }
  }
  *k_out = best_k;
  if (frame_time_out) *frame_time_out = best_t;
  return OXY_OK;
}

int32_t oxy_sched_info(oxy_sched* s, int32_t* frame, int32_t* n_active, int32_t* n_created,
                       int32_t* n_rejected) {
  if (!s) return fail(OXY_ERR_INVALID_ARG, "sched_info: null");
  if (frame) *frame = s->frame;
  if (n_active) *n_active = (int32_t)s->active.size();
  if (n_created) *n_created = s->n_created;
  if (n_rejected) *n_rejected = s->n_rejected;
  return OXY_OK;
}

int32_t oxy_sched_request_info(oxy_sched* s, int32_t request_id, int32_t* stream_id, int32_t* done,
                               int32_t* target, int32_t* birth_frame) {
  if (!s) return fail(OXY_ERR_INVALID_ARG, "sched_request_info: null");
  const Request* r = find_request(s, request_id);
  if (!r) return fail(OXY_ERR_BAD_ID, "sched_request_info: request %d is not active", request_id);
  if (stream_id) *stream_id = r->sid;
  if (done) *done = r->done;
  if (target) *target = r->target;
  if (birth_frame) *birth_frame = r->birth;
  return OXY_OK;
}

}  // extern "C"
