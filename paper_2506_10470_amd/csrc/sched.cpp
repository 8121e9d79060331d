// TD-Pipe control decisions (paper Sec. 3.3 - 3.5) and the simulated pipeline they drive
// (Sec. 3.1): host code, no GPU.  Declared in include/tdp_sched.h.
#include "../../include/tdp_sched.h"

#include <algorithm>
#include <cmath>
#include <deque>
#include <limits>
#include <new>
#include <unordered_set>
#include <vector>

namespace {

constexpr int kDefaultFirst = 32, kDefaultLast = 1024, kDefaultStep = 32;  // Sec. 3.3: steps 32, 64, ..., 1024

struct Profile {
  const double* x;
  const double* ms;
  int n;
  bool ok() const {
    if (!x || !ms || n < 1) return false;
    for (int i = 0; i < n; ++i)
      if (!(x[i] > 0) || !(ms[i] > 0) || (i > 0 && !(x[i] > x[i - 1]))) return false;
    return true;
  }
  double time(double at) const {
    if (at <= x[0]) return ms[0];
    if (at >= x[n - 1]) return ms[n - 1] * (at / x[n - 1]);
    int i = 0;
    while (!(x[i] <= at && at <= x[i + 1])) ++i;
    return ms[i] + (ms[i + 1] - ms[i]) * ((at - x[i]) / (x[i + 1] - x[i]));
  }
  double peak() const {
    double best = 0;
    for (int i = 0; i < n; ++i) best = std::max(best, x[i] / ms[i]);
    return best;
  }
  double spatial(double batch) const { return batch <= 0 ? 0.0 : (batch / time(batch)) / peak(); }
};

double temporal(const double* pending, int n_pending, double decode_ms, int n_batches, bool count_steps) {
  if (n_pending <= 0) return 0.0;
  double longest = pending[0], sum = 0;
  for (int i = 0; i < n_pending; ++i) {
    longest = std::max(longest, pending[i]);
    sum += pending[i];
  }
  const double bubble = std::max(0.0, longest - decode_ms);
  double total = sum + bubble;
  if (count_steps) total += n_batches * decode_ms;
  return 1.0 - bubble / total;
}

}  // namespace

// ---------------------------------------------------------------------------------- Algorithm 1
struct tdp_prefill_switch {
  int64_t capacity;
  std::vector<int32_t> points;  // ascending
  std::vector<int64_t> usage;
  void update(int64_t input_len, int64_t predict_len) {
    for (size_t i = 0; i < points.size() && points[i] <= predict_len; ++i) usage[i] += input_len + points[i];
  }
  bool over() const {
    int64_t mx = 0;
    for (int64_t u : usage) mx = std::max(mx, u);
    return mx > capacity;
  }
};

// ---------------------------------------------------------------------------------- work stealing
struct tdp_work_stealing {
  std::vector<std::vector<int64_t>> batches;
  std::deque<int64_t> withheld;
  int64_t live() const {
    int64_t t = (int64_t)withheld.size();
    for (const auto& b : batches) t += (int64_t)b.size();
    return t;
  }
  const std::vector<int64_t>& on_return(int i, const int64_t* finished, int n_finished) {
    std::vector<int64_t>& b = batches[i];
    if (n_finished > 0) {
      std::unordered_set<int64_t> done(finished, finished + n_finished);
      b.erase(std::remove_if(b.begin(), b.end(), [&](int64_t r) { return done.count(r) != 0; }), b.end());
    }
    const int64_t n = (int64_t)batches.size();
    const int64_t average = (live() + n - 1) / n;
    if ((int64_t)b.size() > average) {
      withheld.insert(withheld.end(), b.begin() + average, b.end());
      b.resize((size_t)average);
    } else {
      while ((int64_t)b.size() < average && !withheld.empty()) {
        b.push_back(withheld.front());
        withheld.pop_front();
      }
    }
    return b;
  }
};

namespace {

tdp_prefill_switch make_switch(int64_t capacity, const int32_t* points, int n_points) {
  tdp_prefill_switch s;
  s.capacity = capacity;
  if (points) s.points.assign(points, points + n_points);
  else
    for (int p = kDefaultFirst; p <= kDefaultLast; p += kDefaultStep) s.points.push_back(p);
  s.usage.assign(s.points.size(), 0);
  return s;
}

tdp_work_stealing make_stealing(int n_batches, const int64_t* ids, int64_t n_ids) {
  tdp_work_stealing w;
  w.batches.resize((size_t)n_batches);
  const int64_t q = n_ids / n_batches, r = n_ids % n_batches;
  int64_t pos = 0;
  for (int i = 0; i < n_batches; ++i) {
    const int64_t size = q + (i < r ? 1 : 0);
    w.batches[(size_t)i].assign(ids + pos, ids + pos + size);
    pos += size;
  }
  return w;
}

int copy_ids(const std::vector<int64_t>& v, int64_t* out, int32_t cap, int32_t* n_out) {
  if (!n_out || cap < 0 || (cap > 0 && !out) || (int64_t)v.size() > cap) return TDP_SCHED_EINVAL;
  std::copy(v.begin(), v.end(), out);
  *n_out = (int32_t)v.size();
  return 0;
}

// ------------------------------------------------------------------------------ simulated pipeline
struct Request {
  int64_t input_len, output_len, predict_len, generated;
};

struct Simulation {
  const tdp_sim_config& cfg;
  Profile dec, pre;
  std::vector<Request> req;
  std::deque<int64_t> waiting;     // request ids, first come first served
  std::vector<int64_t> running;    // live requests in admission order
  std::vector<double> stage_free;
  std::vector<double> ready_at;    // per request: when its newest token became available (its prefill left the pipeline)
  int64_t kv = 0;                  // tokens held by the running requests
  tdp_sim_result res{};
  tdp_sim_event* events = nullptr;
  int64_t events_cap = 0;
  const tdp_sim_executor* exec = nullptr;  // optional: does the work each event stands for
  bool aborted = false;

  Simulation(const tdp_sim_config& c, Profile d, Profile p) : cfg(c), dec(d), pre(p) {}

  struct PlannedBatch {
    int64_t count, tokens;
  };

  void event(int kind, double t, int64_t a, int64_t b) {
    if (res.n_events < events_cap && events) events[res.n_events] = tdp_sim_event{kind, t, a, b};
    ++res.n_events;
  }
  double run_batch(double ready, double dur) {
    double t = ready;
    for (double& free_at : stage_free) {
      const double start = std::max(t, free_at);
      t = start + dur;
      free_at = t;
      res.busy_ms += dur;
    }
    return t;
  }
  // The batches the next prefill phase launches: consecutive runs of the waiting queue.
  std::vector<PlannedBatch> plan_prefill() const {
    tdp_prefill_switch sw = make_switch(cfg.kv_capacity, nullptr, 0);
    int64_t held = 0;
    for (int64_t id : running) {
      const Request& r = req[(size_t)id];
      sw.update(r.input_len + r.generated, std::max<int64_t>(r.predict_len - r.generated, 1));
      held += r.input_len + r.generated;
    }
    std::vector<PlannedBatch> plan;
    size_t pos = 0;
    while (pos < waiting.size()) {
      int64_t count = 0, tokens = 0;
      const size_t first = pos;
      while (pos < waiting.size()) {
        const int64_t len = req[(size_t)waiting[pos]].input_len;
        if (count > 0 && tokens + len > cfg.prefill_token_budget) break;
        if (held + tokens + len + 1 > cfg.kv_capacity) break;  // the prompt itself does not fit now
        ++count;
        tokens += len;
        ++pos;
      }
      if (count == 0) break;
      plan.push_back(PlannedBatch{count, tokens});
      held += tokens + count;  // prompts plus the first generated token of each
      for (size_t p = first; p < pos; ++p) {
        const Request& r = req[(size_t)waiting[p]];
        sw.update(r.input_len, r.predict_len);
      }
      if (cfg.greedy_prefill && sw.over()) break;
    }
    return plan;
  }
  void remove_running(const std::unordered_set<int64_t>& gone) {
    running.erase(std::remove_if(running.begin(), running.end(), [&](int64_t r) { return gone.count(r) != 0; }),
                  running.end());
  }

  bool abort_run() {
    aborted = true;
    return false;
  }

  bool run() {
    const int n = cfg.n_stages;
    stage_free.assign((size_t)n, 0.0);
    double now = 0.0;
    while (!waiting.empty() || !running.empty()) {
      // ---- prefill phase
      const std::vector<PlannedBatch> plan = plan_prefill();
      double last_finish = now;
      for (const PlannedBatch& b : plan) {
        const double finish = run_batch(std::max(now, stage_free[0]), pre.time((double)b.tokens));
        event(0, finish, b.count, b.tokens);
        res.prefill_tokens += b.tokens;
        std::vector<int64_t> ids;
        std::vector<int32_t> lens;
        for (int64_t k = 0; k < b.count; ++k) {
          const int64_t id = waiting.front();
          waiting.pop_front();
          Request& r = req[(size_t)id];
          r.generated = 1;  // the prefill produces the first output token
          ++res.generated_tokens;
          kv += r.input_len + 1;
          running.push_back(id);
          ready_at[(size_t)id] = finish;
          ids.push_back(id);
          lens.push_back((int32_t)r.input_len);
        }
        if (exec && exec->prefill && exec->prefill(exec->user, ids.data(), lens.data(), (int32_t)ids.size()) != 0)
          return abort_run();
        last_finish = std::max(last_finish, finish);
      }
      res.peak_kv_tokens = std::max(res.peak_kv_tokens, kv);
      {  // requests whose only output token came from the prefill are finished already
        std::unordered_set<int64_t> gone;
        for (int64_t id : running)
          if (req[(size_t)id].generated >= req[(size_t)id].output_len) {
            gone.insert(id);
            kv -= req[(size_t)id].input_len + req[(size_t)id].generated;
          }
        if (!gone.empty()) {
          const std::vector<int64_t> ids(gone.begin(), gone.end());
          if (exec && exec->release && exec->release(exec->user, ids.data(), (int32_t)ids.size(), 0) != 0)
            return abort_run();
          remove_running(gone);
        }
      }
      if (running.empty()) {
        if (plan.empty()) return false;  // a prompt does not fit the capacity on its own
        now = last_finish;
        continue;
      }
      ++res.phase_switches;
      // ---- decode phase, entered compactly (Sec. 3.1: phase switches leave minimal bubbles): a batch
      // starts as soon as stage 0 is free and every request in it has the token its prefill produced
      tdp_work_stealing ws = make_stealing(n, running.data(), (int64_t)running.size());
      std::vector<double> return_at((size_t)n, -1.0);  // < 0: not in flight
      auto launch = [&](int i, double ready) {
        return_at[(size_t)i] = run_batch(ready, dec.time((double)ws.batches[(size_t)i].size()));
      };
      for (int i = 0; i < n; ++i)
        if (!ws.batches[(size_t)i].empty()) {
          double ready = now;
          for (int64_t id : ws.batches[(size_t)i]) ready = std::max(ready, ready_at[(size_t)id]);
          launch(i, std::max(ready, stage_free[0]));
        }
      bool draining = false;
      double t_switch = 0.0;
      for (;;) {
        int i = -1;
        for (int k = 0; k < n; ++k)
          if (return_at[(size_t)k] >= 0 && (i < 0 || return_at[(size_t)k] < return_at[(size_t)i])) i = k;
        if (i < 0) break;
        const double t_ret = return_at[(size_t)i];
        return_at[(size_t)i] = -1.0;
        now = t_ret;
        std::vector<int64_t>& batch = ws.batches[(size_t)i];
        const double step_ms = dec.time((double)batch.size());
        if (exec && exec->decode) {
          std::vector<int32_t> context;  // tokens each request holds in the cache before this step
          for (int64_t id : batch) context.push_back((int32_t)(req[(size_t)id].input_len + req[(size_t)id].generated - 1));
          if (exec->decode(exec->user, i, batch.data(), context.data(), (int32_t)batch.size()) != 0) return abort_run();
        }
        std::vector<int64_t> gone;
        for (int64_t id : batch) {
          Request& r = req[(size_t)id];
          ++r.generated;
          ++res.generated_tokens;
          ++kv;
          if (r.generated >= r.output_len) gone.push_back(id);
        }
        res.peak_kv_tokens = std::max(res.peak_kv_tokens, kv);
        std::unordered_set<int64_t> gone_set(gone.begin(), gone.end());
        for (int64_t id : gone) kv -= req[(size_t)id].input_len + req[(size_t)id].generated;
        if (exec && exec->release && !gone.empty() &&
            exec->release(exec->user, gone.data(), (int32_t)gone.size(), 0) != 0)
          return abort_run();
        const size_t n_finished = gone.size();
        // memory overflow: the most recently admitted request of this batch is recomputed later
        for (size_t k = batch.size(); kv > cfg.kv_capacity && k-- > 0;) {
          const int64_t id = batch[k];
          if (gone_set.count(id)) continue;
          Request& r = req[(size_t)id];
          kv -= r.input_len + r.generated;
          r.input_len += r.generated;
          r.output_len -= r.generated;
          r.predict_len = std::max<int64_t>(r.predict_len - r.generated, 1);
          r.generated = 0;
          waiting.push_front(id);
          gone.push_back(id);
          gone_set.insert(id);
          ++res.recomputes;
        }
        if (exec && exec->release && gone.size() > n_finished &&
            exec->release(exec->user, gone.data() + n_finished, (int32_t)(gone.size() - n_finished), 1) != 0)
          return abort_run();
        if (!gone_set.empty()) remove_running(gone_set);
        if (cfg.work_stealing) {
          ws.on_return(i, gone.data(), (int)gone.size());
        } else {
          batch.erase(std::remove_if(batch.begin(), batch.end(), [&](int64_t r) { return gone_set.count(r) != 0; }),
                      batch.end());
        }
        event(1, t_ret, i, (int64_t)batch.size());
        if (draining) continue;
        if (cfg.intensity_switch && !waiting.empty() && !running.empty() && !batch.empty()) {
          const std::vector<PlannedBatch> pending = plan_prefill();
          if (!pending.empty()) {
            std::vector<double> pend_ms;
            for (const PlannedBatch& b : pending) pend_ms.push_back(pre.time((double)b.tokens));
            if (dec.spatial((double)batch.size()) <
                temporal(pend_ms.data(), (int)pend_ms.size(), step_ms, n, cfg.count_decode_steps != 0)) {
              draining = true;  // the steps in flight come back, nothing is resubmitted
              t_switch = t_ret;
              event(2, t_ret, (int64_t)batch.size(), (int64_t)pend_ms.size());
              continue;
            }
          }
        }
        if (!batch.empty()) launch(i, t_ret);
        if (cfg.work_stealing) {
          // a batch that ran empty earlier is revived as soon as withheld requests exist
          std::vector<char> idle((size_t)n);
          for (int k = 0; k < n; ++k) idle[(size_t)k] = return_at[(size_t)k] < 0;
          for (int k = 0; k < n; ++k)
            if (idle[(size_t)k] && !ws.withheld.empty()) {
              ws.on_return(k, nullptr, 0);
              if (!ws.batches[(size_t)k].empty()) launch(k, t_ret);
            }
        }
      }
      if (draining) {
        ++res.phase_switches;
        // the prefills enter stage 0 behind the steps still in flight instead of waiting for them to return:
        // the bubble of the switch is the mismatch of step times (Sec. 3.5), not a drained pipeline
        now = t_switch;
      }
    }
    res.total_ms = *std::max_element(stage_free.begin(), stage_free.end());
    return true;
  }
};

}  // namespace

extern "C" {

int tdp_sched_abi_version(void) { return 1; }

int tdp_prefill_switch_create(int64_t kv_capacity, const int32_t* future_points, int32_t n_points,
                              tdp_prefill_switch** out) {
  if (!out || kv_capacity < 0) return TDP_SCHED_EINVAL;
  if (future_points) {
    if (n_points < 1) return TDP_SCHED_EINVAL;
    for (int i = 0; i < n_points; ++i)
      if (future_points[i] < 1 || (i > 0 && future_points[i] <= future_points[i - 1])) return TDP_SCHED_EINVAL;
  }
  tdp_prefill_switch* s = new (std::nothrow) tdp_prefill_switch(make_switch(kv_capacity, future_points, n_points));
  if (!s) return TDP_SCHED_EINVAL;
  *out = s;
  return 0;
}
void tdp_prefill_switch_destroy(tdp_prefill_switch* s) { delete s; }
int tdp_prefill_switch_reset(tdp_prefill_switch* s) {
  if (!s) return TDP_SCHED_EINVAL;
  std::fill(s->usage.begin(), s->usage.end(), 0);
  return 0;
}
int tdp_prefill_switch_update(tdp_prefill_switch* s, int32_t input_len, int32_t predict_len) {
  if (!s || input_len < 0 || predict_len < 0) return TDP_SCHED_EINVAL;
  s->update(input_len, predict_len);
  return 0;
}
int tdp_prefill_switch_usage(const tdp_prefill_switch* s, int64_t* usage_out, int32_t n) {
  if (!s || !usage_out || n < (int32_t)s->usage.size()) return TDP_SCHED_EINVAL;
  std::copy(s->usage.begin(), s->usage.end(), usage_out);
  return (int)s->usage.size();
}
int tdp_prefill_switch_check(const tdp_prefill_switch* s) {
  if (!s) return TDP_SCHED_EINVAL;
  return s->over() ? 1 : 0;
}

int tdp_work_stealing_create(int32_t n_batches, const int64_t* request_ids, int32_t n_requests,
                             tdp_work_stealing** out) {
  if (!out || n_batches < 1 || n_requests < 0 || (n_requests > 0 && !request_ids)) return TDP_SCHED_EINVAL;
  tdp_work_stealing* w = new (std::nothrow) tdp_work_stealing(make_stealing(n_batches, request_ids, n_requests));
  if (!w) return TDP_SCHED_EINVAL;
  *out = w;
  return 0;
}
void tdp_work_stealing_destroy(tdp_work_stealing* w) { delete w; }
int tdp_work_stealing_batch(const tdp_work_stealing* w, int32_t batch, int64_t* ids_out, int32_t cap,
                            int32_t* n_out) {
  if (!w || batch < 0 || batch >= (int32_t)w->batches.size()) return TDP_SCHED_EINVAL;
  return copy_ids(w->batches[(size_t)batch], ids_out, cap, n_out);
}
int tdp_work_stealing_withheld(const tdp_work_stealing* w, int64_t* ids_out, int32_t cap, int32_t* n_out) {
  if (!w) return TDP_SCHED_EINVAL;
  return copy_ids(std::vector<int64_t>(w->withheld.begin(), w->withheld.end()), ids_out, cap, n_out);
}
int tdp_work_stealing_on_return(tdp_work_stealing* w, int32_t batch, const int64_t* finished_ids,
                                int32_t n_finished, int64_t* ids_out, int32_t cap, int32_t* n_out) {
  if (!w || batch < 0 || batch >= (int32_t)w->batches.size() || n_finished < 0 || (n_finished > 0 && !finished_ids) ||
      !n_out || cap < 0 || (cap > 0 && !ids_out))
    return TDP_SCHED_EINVAL;
  // the new composition is never larger than what the batch held plus what was withheld
  if ((int64_t)w->batches[(size_t)batch].size() + (int64_t)w->withheld.size() > cap) return TDP_SCHED_EINVAL;
  return copy_ids(w->on_return(batch, finished_ids, n_finished), ids_out, cap, n_out);
}

double tdp_profile_time(const double* x, const double* ms, int32_t n, double at) {
  const Profile p{x, ms, n};
  if (!p.ok() || !(at == at)) return std::numeric_limits<double>::quiet_NaN();
  return p.time(at);
}
double tdp_spatial_intensity(const double* x, const double* ms, int32_t n, double batch) {
  const Profile p{x, ms, n};
  if (!p.ok() || !(batch == batch)) return std::numeric_limits<double>::quiet_NaN();
  return p.spatial(batch);
}
double tdp_temporal_intensity(const double* pending_prefill_ms, int32_t n_pending, double decode_ms,
                              int32_t n_batches, int32_t count_decode_steps) {
  if (n_pending < 0 || (n_pending > 0 && !pending_prefill_ms) || !(decode_ms >= 0) || n_batches < 1)
    return std::numeric_limits<double>::quiet_NaN();
  return temporal(pending_prefill_ms, n_pending, decode_ms, n_batches, count_decode_steps != 0);
}
int tdp_switch_to_prefill(const double* x, const double* ms, int32_t n, double batch,
                          const double* pending_prefill_ms, int32_t n_pending, double decode_ms, int32_t n_batches,
                          int32_t count_decode_steps) {
  const double s = tdp_spatial_intensity(x, ms, n, batch);
  const double t = tdp_temporal_intensity(pending_prefill_ms, n_pending, decode_ms, n_batches, count_decode_steps);
  if (!(s == s) || !(t == t)) return TDP_SCHED_EINVAL;
  return s < t ? 1 : 0;
}

int tdp_simulate_exec(const tdp_sim_config* cfg, const int32_t* input_len, const int32_t* output_len,
                      const int32_t* predict_len, int64_t n_requests, const double* decode_x, const double* decode_ms,
                      int32_t n_decode, const double* prefill_x, const double* prefill_ms, int32_t n_prefill,
                      tdp_sim_result* result, tdp_sim_event* events, int64_t events_cap,
                      const tdp_sim_executor* exec) {
  if (!cfg || !result || n_requests < 0 || (n_requests > 0 && (!input_len || !output_len || !predict_len)) ||
      events_cap < 0 || (events_cap > 0 && !events))
    return TDP_SCHED_EINVAL;
  if (cfg->n_stages < 1 || cfg->kv_capacity < 1 || cfg->prefill_token_budget < 1) return TDP_SCHED_EINVAL;
  Simulation sim(*cfg, Profile{decode_x, decode_ms, n_decode}, Profile{prefill_x, prefill_ms, n_prefill});
  if (!sim.dec.ok() || !sim.pre.ok()) return TDP_SCHED_EINVAL;
  sim.events = events;
  sim.events_cap = events_cap;
  sim.exec = exec;
  sim.req.resize((size_t)n_requests);
  sim.ready_at.assign((size_t)n_requests, 0.0);
  for (int64_t i = 0; i < n_requests; ++i) {
    if (input_len[i] < 1 || output_len[i] < 1 || predict_len[i] < 0) return TDP_SCHED_EINVAL;
    sim.req[(size_t)i] = Request{input_len[i], output_len[i], predict_len[i], 0};
    sim.waiting.push_back(i);
  }
  if (!sim.run()) return sim.aborted ? TDP_SCHED_EABORT : TDP_SCHED_EINVAL;
  *result = sim.res;
  return 0;
}

int tdp_simulate(const tdp_sim_config* cfg, const int32_t* input_len, const int32_t* output_len,
                 const int32_t* predict_len, int64_t n_requests, const double* decode_x, const double* decode_ms,
                 int32_t n_decode, const double* prefill_x, const double* prefill_ms, int32_t n_prefill,
                 tdp_sim_result* result, tdp_sim_event* events, int64_t events_cap) {
  return tdp_simulate_exec(cfg, input_len, output_len, predict_len, n_requests, decode_x, decode_ms, n_decode,
                           prefill_x, prefill_ms, n_prefill, result, events, events_cap, nullptr);
}

}  // extern "C"
