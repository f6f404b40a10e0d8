// Host side of the adapter scheduler (Sec. 3.4, Algorithm 1 Phase 1 and the outer loop on one device): grouping
// of jobs over a measured step-time model.  Plain C++; no device code.  All arithmetic is IEEE double in a fixed
// order with contraction off, so that decisions are reproducible bit for bit.
#pragma clang fp contract(off)
#include <algorithm>
#include <cstdint>
#include <vector>

#include "../../include/tlora.h"

namespace {

struct Model {
  const tlora_sched_model_t* m;
  double curve(int64_t tokens) const {
    const double t = (double)tokens;
    const double* xs = m->tokens;
    const double* ys = m->ms;
    if (t <= xs[0]) return ys[0];
    int i = m->n_points - 2;
    for (int k = 0; k + 1 < m->n_points; ++k)
      if (t < xs[k + 1]) { i = k;  break; }
    return ys[i] + (ys[i + 1] - ys[i]) * ((t - xs[i]) / (xs[i + 1] - xs[i]));
  }
  double peak() const {
    double best = 0.0;
    for (int i = 0; i < m->n_points; ++i) best = std::max(best, m->tokens[i] / m->ms[i]);
    return best;
  }
};

typedef std::vector<int32_t> Group;      // sorted job indices

struct Ctx {
  Model model;
  const tlora_sched_job_t* jobs;
  double pk;
  int64_t tokens(const Group& g) const {
    int64_t t = 0;
    for (int32_t j : g) t += jobs[j].tokens;
    return t;
  }
  double step_ms(const Group& g) const {
    int64_t total = 0;
    double work = 0.0;
    for (int32_t j : g) {
      total += jobs[j].tokens;
      work += (double)jobs[j].tokens * (double)jobs[j].rank;
    }
    return model.curve(total) + model.m->ms_per_token_rank * work + model.m->ms_per_job * (double)((int64_t)g.size() - 1);
  }
  double step_ms1(int32_t j) const { return step_ms(Group{j}); }
  double throughput(const Group& g) const { return (double)tokens(g) / step_ms(g); }
  double residual(const Group& g) const { return 1.0 - throughput(g) / pk; }
  bool feasible(const Group& g) const {
    const double t = step_ms(g);
    for (int32_t j : g)
      if (!(t / step_ms1(j) <= jobs[j].max_slowdown)) return false;
    return true;
  }
};

struct Item {
  Group members;
  double urgency, residual;
};

Group merged(const Group& a, const Group& b) {
  Group u(a);
  u.insert(u.end(), b.begin(), b.end());
  std::sort(u.begin(), u.end());
  return u;
}

Item make_item(const Ctx& c, const std::vector<double>& urgency, Group g) {
  Item it;
  it.urgency = urgency[g[0]];
  for (int32_t j : g) it.urgency = std::max(it.urgency, urgency[j]);
  it.residual = c.residual(g);
  it.members = std::move(g);
  return it;
}

// One pass of Phase 1 over the queue `active`: the finalized group.
Group next_group(const Ctx& c, const std::vector<int32_t>& active, const std::vector<double>& urgency) {
  std::vector<Item> items;
  for (int32_t j : active) items.push_back(make_item(c, urgency, Group{j}));
  for (;;) {
    std::stable_sort(items.begin(), items.end(), [](const Item& a, const Item& b) {
      if (a.urgency != b.urgency) return a.urgency > b.urgency;
      if (a.residual != b.residual) return a.residual < b.residual;
      return a.members[0] < b.members[0];
    });
    const Item& seed = items[0];
    int best = -1;
    double best_thr = 0.0;
    const double seed_ms = c.step_ms(seed.members);
    for (size_t k = 1; k < items.size(); ++k) {
      const Group u = merged(seed.members, items[k].members);
      if (!c.feasible(u)) continue;
      const double thr = c.throughput(u);
      const double shared = (double)c.tokens(u) / (seed_ms + c.step_ms(items[k].members));
      if (!(thr > shared)) continue;
      if (best < 0 || thr > best_thr) { best = (int)k;  best_thr = thr; }
    }
    if (best < 0) return seed.members;
    Item m = make_item(c, urgency, merged(seed.members, items[best].members));
    std::vector<Item> next;
    for (size_t k = 1; k < items.size(); ++k)
      if ((int)k != best) next.push_back(std::move(items[k]));
    next.push_back(std::move(m));
    items.swap(next);
  }
}

int check(const tlora_sched_model_t* m, int32_t n_jobs, const tlora_sched_job_t* jobs) {
  if (!m || !m->tokens || !m->ms || (n_jobs > 0 && !jobs)) return TLORA_ENULL;
  if (m->n_points < 2 || n_jobs < 0 || !(m->ms_per_token_rank >= 0.0) || !(m->ms_per_job >= 0.0))
    return TLORA_EINVAL;
  for (int i = 0; i < m->n_points; ++i) {
    if (!(m->tokens[i] > 0.0) || !(m->ms[i] > 0.0)) return TLORA_EINVAL;
    if (i && !(m->tokens[i] > m->tokens[i - 1])) return TLORA_EINVAL;
  }
  for (int32_t j = 0; j < n_jobs; ++j)
    if (jobs[j].tokens < 1 || jobs[j].rank < 0 || !(jobs[j].max_slowdown >= 1.0) || !(jobs[j].urgency >= 0.0) ||
        jobs[j].steps < 0)
      return TLORA_EINVAL;
  return TLORA_OK;
}

}  // namespace

extern "C" {

int tlora_sched_step_ms(const tlora_sched_model_t* model, int32_t n_jobs, const tlora_sched_job_t* jobs,
                        const int32_t* members, int32_t n_members, double* ms) {
  int rc = check(model, n_jobs, jobs);
  if (rc != TLORA_OK) return rc;
  if (!ms || (n_members > 0 && !members)) return TLORA_ENULL;
  if (n_members < 1) return TLORA_EINVAL;
  Group g;
  for (int32_t i = 0; i < n_members; ++i) {
    if (members[i] < 0 || members[i] >= n_jobs) return TLORA_EINVAL;
    g.push_back(members[i]);
  }
  const Ctx c{Model{model}, jobs, Model{model}.peak()};
  *ms = c.step_ms(g);
  return TLORA_OK;
}

int tlora_sched_partition(const tlora_sched_model_t* model, int32_t n_jobs, const tlora_sched_job_t* jobs,
                          int32_t* group_of, int32_t* n_groups) {
  int rc = check(model, n_jobs, jobs);
  if (rc != TLORA_OK) return rc;
  if (!n_groups || (n_jobs > 0 && !group_of)) return TLORA_ENULL;
  const Ctx c{Model{model}, jobs, Model{model}.peak()};
  std::vector<double> urgency(n_jobs);
  std::vector<int32_t> active(n_jobs);
  for (int32_t j = 0; j < n_jobs; ++j) { urgency[j] = jobs[j].urgency;  active[j] = j; }
  int32_t g = 0;
  while (!active.empty()) {
    const Group grp = next_group(c, active, urgency);
    for (int32_t j : grp) group_of[j] = g;
    std::vector<int32_t> rest;
    for (int32_t j : active)
      if (!std::binary_search(grp.begin(), grp.end(), j)) rest.push_back(j);
    active.swap(rest);
    ++g;
  }
  *n_groups = g;
  return TLORA_OK;
}

int tlora_sched_simulate(const tlora_sched_model_t* model, int32_t n_jobs, const tlora_sched_job_t* jobs, int32_t horizon,
                         double* jct_ms, double* makespan_ms, int32_t* trace_members, int32_t* trace_sizes,
                         int32_t* trace_steps, int64_t* n_rounds, int64_t trace_capacity) {
  int rc = check(model, n_jobs, jobs);
  if (rc != TLORA_OK) return rc;
  if (horizon < 1) return TLORA_EINVAL;
  if (!makespan_ms || !n_rounds || (n_jobs > 0 && !jct_ms)) return TLORA_ENULL;
  const Ctx c{Model{model}, jobs, Model{model}.peak()};
  std::vector<int64_t> left(n_jobs), done(n_jobs, 0);
  std::vector<double> alone(n_jobs), urgency(n_jobs, 1.0);
  std::vector<int32_t> active;
  for (int32_t j = 0; j < n_jobs; ++j) {
    left[j] = jobs[j].steps;
    alone[j] = c.step_ms1(j);
    jct_ms[j] = 0.0;
    if (left[j] > 0) active.push_back(j);
  }
  double now = 0.0;
  int64_t rounds = 0, written = 0;
  while (!active.empty()) {
    std::fill(urgency.begin(), urgency.end(), 1.0);
    for (int32_t j : active)
      if (now > 0.0) urgency[j] = now / (alone[j] * (double)std::max<int64_t>(done[j], 1));
    const Group g = next_group(c, active, urgency);
    int64_t steps = horizon;
    for (int32_t j : g) steps = std::min(steps, left[j]);
    now = now + (double)steps * c.step_ms(g);
    for (int32_t j : g) {
      left[j] -= steps;
      done[j] += steps;
      if (left[j] == 0) jct_ms[j] = now;
    }
    if (trace_members && trace_sizes && trace_steps && rounds < trace_capacity &&
        written + (int64_t)g.size() <= trace_capacity * (int64_t)std::max(n_jobs, 1)) {
      for (int32_t j : g) trace_members[written++] = j;
      trace_sizes[rounds] = (int32_t)g.size();
      trace_steps[rounds] = (int32_t)steps;
    }
    ++rounds;
    std::vector<int32_t> rest;
    for (int32_t j : active)
      if (left[j] > 0) rest.push_back(j);
    active.swap(rest);
  }
  *makespan_ms = now;
  *n_rounds = rounds;
  return TLORA_OK;
}

}  // extern "C"
