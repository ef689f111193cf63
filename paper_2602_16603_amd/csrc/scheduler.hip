// Event-driven scheduler of FlowPrefill Section 5.2: the S-EDF priority of Eq. (3), SLO-aware
// batching (Algorithm 1) and the scheduling round of Algorithm 2, as host-side bookkeeping behind
// fp_sched_*.  No device code: the caller turns decisions into fp_prefill_* / fp_preempt /
// fp_resume calls.
#include <algorithm>
#include <cstdio>
#include <unordered_map>
#include <vector>

#include "../../include/flowprefill.h"
#include "kernels.h"

namespace {

enum State : int { kWaiting = 0, kPreempted = 1, kRunning = 2 };

struct Entry {
  int64_t id;
  int64_t tokens;                 // aggregate of the batch once this request heads one
  double arrival, deadline;
  State state;
  std::vector<int64_t> members;   // requests executed under this head (head included)
};

fp_status sched_fail(fp_status code, const char* text) {
  fp::set_last_error(text);
  return code;
}

}  // namespace

struct fp_sched {
  int64_t budget = 0;
  std::vector<double> coef;
  int32_t policy = FP_SCHED_SEDF;
  bool batching = true;
  std::unordered_map<int64_t, Entry> live;   // Q_w, Q_p and E together
  int64_t running = -1;                       // E

  double predict(int64_t n) const {           // Horner
    double y = 0.0;
    for (size_t i = coef.size(); i-- > 0;) y = y * (double)n + coef[i];
    return y;
  }
  // Larger is more urgent.
  double priority(const Entry& e, double now) const {
    switch (policy) {
      case FP_SCHED_SEDF: {
        const double slack = e.deadline - now - predict(e.tokens);
        return (slack >= 0.0 ? 1.0 : -1.0) / e.deadline;      // Eq. (3), sgn(0) = +1
      }
      case FP_SCHED_EDF: return 1.0 / e.deadline;
      default: return -e.arrival;
    }
  }
};

extern "C" {

fp_status fp_sched_create(int64_t token_budget, const double* ttft_coef, int32_t n_coef,
                          int32_t policy, int32_t batching, fp_sched** out) {
  if (!out || !ttft_coef || n_coef <= 0 || n_coef > 8 || token_budget <= 0 || policy < FP_SCHED_SEDF ||
      policy > FP_SCHED_FCFS)
    return sched_fail(FP_ERR_INVALID, "fp_sched_create: bad argument");
  fp_sched* s = new fp_sched;
  s->budget = token_budget;
  s->coef.assign(ttft_coef, ttft_coef + n_coef);
  s->policy = policy;
  s->batching = batching != 0;
  *out = s;
  return FP_OK;
}

void fp_sched_destroy(fp_sched* sched) { delete sched; }

fp_status fp_sched_arrive(fp_sched* sched, int64_t id, int64_t n_tokens, double arrival,
                          double ttft_slo) {
  if (!sched || id < 0 || n_tokens <= 0 || !(ttft_slo > 0.0) || !(arrival + ttft_slo > 0.0))
    return sched_fail(FP_ERR_INVALID, "fp_sched_arrive: bad argument (ids >= 0, tokens > 0, deadline > 0)");
  if (sched->live.count(id)) return sched_fail(FP_ERR_STATE, "fp_sched_arrive: id already queued");
  sched->live.emplace(id, Entry{id, n_tokens, arrival, arrival + ttft_slo, kWaiting, {id}});
  return FP_OK;
}

fp_status fp_sched_complete(fp_sched* sched, int64_t head_id) {
  if (!sched) return sched_fail(FP_ERR_INVALID, "fp_sched_complete: null scheduler");
  if (sched->running != head_id || head_id < 0)
    return sched_fail(FP_ERR_STATE, "fp_sched_complete: that execution is not the running one");
  sched->live.erase(head_id);
  sched->running = -1;
  return FP_OK;
}

fp_status fp_sched_retire(fp_sched* sched, int64_t id) {
  if (!sched) return sched_fail(FP_ERR_INVALID, "fp_sched_retire: null scheduler");
  auto it = sched->live.find(id);
  if (it == sched->live.end() || it->second.state != kPreempted)
    return sched_fail(FP_ERR_STATE, "fp_sched_retire: that execution is not in the preempted queue");
  sched->live.erase(it);
  return FP_OK;
}

fp_status fp_sched_round(fp_sched* sched, double now, fp_sched_decision* d) {
  if (!sched || !d) return sched_fail(FP_ERR_INVALID, "fp_sched_round: null argument");
  d->preempt_id = -1;
  d->action = FP_SCHED_NONE;
  d->n_batch = 0;
  d->head_id = -1;
  if (sched->live.empty()) return FP_OK;
  if (sched->policy == FP_SCHED_FCFS && sched->running >= 0) return FP_OK;   // never preempts

  // Q_all ranked by descending priority; ties: earlier arrival, then smaller id.
  struct Ranked { double prio; double arrival; int64_t id; };
  std::vector<Ranked> order;
  order.reserve(sched->live.size());
  for (const auto& kv : sched->live)
    order.push_back({sched->priority(kv.second, now), kv.second.arrival, kv.first});
  std::sort(order.begin(), order.end(), [](const Ranked& a, const Ranked& b) {
    if (a.prio != b.prio) return a.prio > b.prio;
    if (a.arrival != b.arrival) return a.arrival < b.arrival;
    return a.id < b.id;
  });
  Entry& head = sched->live.at(order[0].id);
  if (head.id == sched->running) return FP_OK;

  std::vector<int64_t> batch;
  if (head.state == kWaiting) {
    // Algorithm 1: admit waiting requests, in priority order, while the head's remaining time
    // covers the predicted latency of the grown batch and the token budget is not reached.
    batch.push_back(head.id);
    if (sched->batching) {
      const double t_remain = head.deadline - now;
      int64_t n_total = head.tokens;
      for (size_t i = 1; i < order.size() && (int)batch.size() < FP_SCHED_MAX_BATCH; ++i) {
        const Entry& r = sched->live.at(order[i].id);
        if (r.state != kWaiting) continue;
        const int64_t n = n_total + r.tokens;
        if (t_remain > sched->predict(n) && n < sched->budget) {
          batch.push_back(r.id);
          n_total = n;
        }
      }
      head.tokens = n_total;
    }
  }
  if (sched->running >= 0) {
    d->preempt_id = sched->running;
    sched->live.at(sched->running).state = kPreempted;
  }
  if (!batch.empty()) {
    d->action = FP_SCHED_SUBMIT;
    d->n_batch = (int32_t)batch.size();
    for (size_t i = 0; i < batch.size(); ++i) d->batch_ids[i] = batch[i];
    head.members = batch;
    for (size_t i = 1; i < batch.size(); ++i) sched->live.erase(batch[i]);   // they ride with the head now
  } else {
    d->action = FP_SCHED_RESUME;
  }
  d->head_id = head.id;
  head.state = kRunning;
  sched->running = head.id;
  return FP_OK;
}

double fp_sched_predict(const fp_sched* sched, int64_t n_tokens) {
  return sched ? sched->predict(n_tokens) : 0.0;
}

}  // extern "C"
