// Inter-request scheduling (paper Section 3.2): a binary linear cost model - loading time as a
// linear function of the context tokens to load, computation time as a linear function of the query
// tokens - and the queue policies built on it: shortest-job-first on the modelled prefill cost
// (average TTFT) and least-slack-time-first, LST = DDL - T_load - T_comp (SLO attainment), with the
// policies the paper compares against (FIFO, SJF on the prefill token count, earliest deadline
// first; Section 4.3).  Host code only.  See include/calvo.h for the contract.
#include <cmath>
#include <cstdint>
#include <limits>
#include <vector>

#include "../../include/calvo.h"

namespace {

struct Key {          // smaller is served first; ties: earlier arrival, then lower index
  double priority;
  double arrival;
  int index;
  bool operator<(const Key& o) const {
    if (priority != o.priority) return priority < o.priority;
    if (arrival != o.arrival) return arrival < o.arrival;
    return index < o.index;
  }
};

double model_load(const calvo_cost_model& m, const calvo_job& j) {
  return j.ctx_tokens > 0 ? m.load_per_token_s * (double)j.ctx_tokens + m.load_fixed_s : 0.0;
}
double model_comp(const calvo_cost_model& m, const calvo_job& j) {
  return j.query_tokens > 0 ? m.comp_per_token_s * (double)j.query_tokens + m.comp_fixed_s : 0.0;
}

bool priority_of(int policy, const calvo_cost_model* m, const calvo_job& j, double* out) {
  switch (policy) {
    case CALVO_POLICY_FIFO: *out = j.arrival_s; return true;
    case CALVO_POLICY_SJF: *out = model_load(*m, j) + model_comp(*m, j); return true;
    case CALVO_POLICY_SJF_PT: *out = (double)j.query_tokens; return true;
    case CALVO_POLICY_LSTF: *out = j.deadline_s - model_load(*m, j) - model_comp(*m, j); return true;
    case CALVO_POLICY_EDF: *out = j.deadline_s; return true;
    default: return false;
  }
}

bool needs_model(int policy) { return policy == CALVO_POLICY_SJF || policy == CALVO_POLICY_LSTF; }

int pick(int policy, const calvo_cost_model* m, const calvo_job* jobs, const unsigned char* done, int n, double now) {
  int best = -1;
  Key bk{};
  for (int i = 0; i < n; i++) {
    if ((done && done[i]) || !(jobs[i].arrival_s <= now)) continue;
    Key k{0.0, jobs[i].arrival_s, i};
    priority_of(policy, m, jobs[i], &k.priority);
    if (best < 0 || k < bk) { best = i; bk = k; }
  }
  return best;
}

bool valid_jobs(const calvo_job* jobs, int n) {
  for (int i = 0; i < n; i++)
    if (!std::isfinite(jobs[i].arrival_s) || std::isnan(jobs[i].deadline_s) || jobs[i].ctx_tokens < 0 || jobs[i].query_tokens < 0)
      return false;
  return true;
}

}  // namespace

extern "C" {

int calvo_cost_fit(const double* tokens, const double* seconds, int n, double* per_token_s, double* fixed_s) {
  if (!tokens || !seconds || !per_token_s || !fixed_s || n < 2) return CALVO_EINVAL;
  double mx = 0.0, my = 0.0;
  for (int i = 0; i < n; i++) { mx += tokens[i]; my += seconds[i]; }
  mx /= n; my /= n;
  double sxx = 0.0, sxy = 0.0;
  for (int i = 0; i < n; i++) { sxx += (tokens[i] - mx) * (tokens[i] - mx); sxy += (tokens[i] - mx) * (seconds[i] - my); }
  if (!(sxx > 0.0) || !std::isfinite(sxy)) return CALVO_EINVAL;   // all samples at the same token count
  *per_token_s = sxy / sxx;
  *fixed_s = my - *per_token_s * mx;
  return CALVO_OK;
}

int calvo_cost_estimate(const calvo_cost_model* model, const calvo_job* job, double* load_s, double* comp_s) {
  if (!model || !job || !load_s || !comp_s) return CALVO_EINVAL;
  *load_s = model_load(*model, *job);
  *comp_s = model_comp(*model, *job);
  return CALVO_OK;
}

int calvo_sched_pick(int policy, const calvo_cost_model* model, const calvo_job* jobs, const unsigned char* done, int n,
                     double now, int* out_index) {
  if (!out_index || n < 0 || (n > 0 && !jobs) || (needs_model(policy) && !model)) return CALVO_EINVAL;
  if (policy < CALVO_POLICY_FIFO || policy > CALVO_POLICY_EDF) return CALVO_EINVAL;
  if (!valid_jobs(jobs, n)) return CALVO_EINVAL;
  *out_index = pick(policy, model, jobs, done, n, now);
  return CALVO_OK;
}

int calvo_sched_simulate(int policy, const calvo_cost_model* model, const calvo_job* jobs, int n, const double* load_s,
                         const double* comp_s, int pipelined, double* start_s, double* finish_s) {
  if (n < 0 || (n > 0 && (!jobs || !start_s || !finish_s))) return CALVO_EINVAL;
  if (policy < CALVO_POLICY_FIFO || policy > CALVO_POLICY_EDF) return CALVO_EINVAL;
  if ((needs_model(policy) || !load_s || !comp_s) && !model) return CALVO_EINVAL;
  if (!valid_jobs(jobs, n)) return CALVO_EINVAL;
  if (pipelined < 0 || pipelined > 2) return CALVO_EINVAL;
  for (int i = 0; i < n; i++) {                        // measured times must be finite and non-negative
    if (load_s && !(load_s[i] >= 0.0 && std::isfinite(load_s[i]))) return CALVO_EINVAL;
    if (comp_s && !(comp_s[i] >= 0.0 && std::isfinite(comp_s[i]))) return CALVO_EINVAL;
  }
  std::vector<unsigned char> done((size_t)n, 0);
  double loader_free = -std::numeric_limits<double>::infinity();
  double compute_free = -std::numeric_limits<double>::infinity();
  if (pipelined == 2) {
    // Two stages that each serve their highest-priority ready request (Section 3.1): the loading
    // stage picks among the requests that have arrived, the compute stage among those whose loading
    // has finished; decisions in time order, the compute stage first at equal times.
    const double inf = std::numeric_limits<double>::infinity();
    std::vector<unsigned char> taken((size_t)n, 0);
    std::vector<double> load_end((size_t)n, inf);
    for (int step = 0; step < 2 * n; step++) {
      double t_l = inf, t_c = inf, first_arrival = inf, first_ready = inf;
      for (int i = 0; i < n; i++) {
        if (!taken[i] && jobs[i].arrival_s < first_arrival) first_arrival = jobs[i].arrival_s;
        if (taken[i] && !done[i] && load_end[i] < first_ready) first_ready = load_end[i];
      }
      if (first_arrival < inf) t_l = loader_free > first_arrival ? loader_free : first_arrival;
      if (first_ready < inf) t_c = compute_free > first_ready ? compute_free : first_ready;
      if (t_c <= t_l) {
        int best = -1;
        Key bk{};
        for (int i = 0; i < n; i++) {
          if (!taken[i] || done[i] || !(load_end[i] <= t_c)) continue;
          Key k{0.0, jobs[i].arrival_s, i};
          priority_of(policy, model, jobs[i], &k.priority);
          if (best < 0 || k < bk) { best = i; bk = k; }
        }
        if (best < 0) return CALVO_EINVAL;             // cannot happen with finite times
        finish_s[best] = t_c + (comp_s ? comp_s[best] : model_comp(*model, jobs[best]));
        compute_free = finish_s[best];
        done[best] = 1;
      } else {
        const int i = pick(policy, model, jobs, taken.data(), n, t_l);
        start_s[i] = t_l;
        load_end[i] = t_l + (load_s ? load_s[i] : model_load(*model, jobs[i]));
        loader_free = load_end[i];
        taken[i] = 1;
      }
    }
    return CALVO_OK;
  }
  for (int served = 0; served < n; served++) {
    // the server (its loading stage, when pipelined) takes the next job when it is free and a job
    // has arrived; otherwise it idles until the next arrival
    const double free_at = pipelined ? loader_free : compute_free;
    double next_arrival = std::numeric_limits<double>::infinity();
    for (int i = 0; i < n; i++)
      if (!done[i] && jobs[i].arrival_s < next_arrival) next_arrival = jobs[i].arrival_s;
    const double now = free_at > next_arrival ? free_at : next_arrival;
    const int i = pick(policy, model, jobs, done.data(), n, now);
    const double tl = load_s ? load_s[i] : model_load(*model, jobs[i]);
    const double tc = comp_s ? comp_s[i] : model_comp(*model, jobs[i]);
    start_s[i] = now;
    const double load_end = now + tl;
    const double comp_start = (pipelined && compute_free > load_end) ? compute_free : load_end;
    finish_s[i] = comp_start + tc;
    loader_free = load_end;
    compute_free = finish_s[i];
    done[i] = 1;
  }
  return CALVO_OK;
}

}  // extern "C"
