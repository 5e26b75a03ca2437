// Host side of OTAS behind the C ABI of include/otas_sched.h: the batch queue with adaptive batching
// (Sec. III-C, Alg. 1) and online token adaptation (Sec. III-D, Alg. 2 / Alg. 3 and the profile-based
// estimates).  Pure host code: no device call anywhere in this file.
//
// Layout: a batch keeps the aggregates the algorithms ask for (earliest arrival, earliest deadline, first
// utility, utility sum, per-task request counts) up to date as requests join, so Alg. 1 is O(batches
// walked) per request and a profile estimate is O(tasks) for the time and O(batch) for the utility.  The
// dynamic program evaluates every (batch, gamma) estimate once, keeps two rolling rows of accumulated
// utility and clock, and stores only the predecessor table for the backtracking.
#include <algorithm>
#include <cmath>
#include <cstdint>
#include <limits>
#include <new>
#include <vector>

#include "../../include/otas.h"
#include "../../include/otas_sched.h"

namespace {

struct Request {
  int64_t id;
  double u;
  int32_t task;
};

struct Batch {
  std::vector<Request> req;        // arrival order
  std::vector<int32_t> per_task;   // request count of each task
  double s_b, d_b, u_first, u_sum;
  int32_t gamma;                   // index into gammas, OTAS_GAMMA_SKIP or OTAS_GAMMA_UNDECIDED
};

}  // namespace

struct otas_sched {
  otas_sched_params p;
  int32_t NG, NT;
  std::vector<int32_t> gammas;
  std::vector<double> latency, accuracy;     // [task][gamma index]
  std::vector<double> rate_max;
  std::vector<int32_t> rate_gamma;
  int32_t g_smallest, g_largest;
  std::vector<Batch> queue;

  double time_of(const Batch& b, int32_t g) const {
    double t = 0.0;
    for (int32_t k = 0; k < NT; ++k) t += b.per_task[k] * latency[(size_t)k * NG + g];
    return t;
  }
  double utility_of(const Batch& b, int32_t g) const {
    double U = 0.0;
    for (const Request& r : b.req) U += r.u * accuracy[(size_t)r.task * NG + g];
    return U;
  }
  int32_t gamma_for_rate(double q) const {
    for (size_t i = 0; i < rate_max.size(); ++i)
      if (q <= rate_max[i]) return rate_gamma[i];
    return g_smallest;
  }

  // Alg. 3 over the (already sorted) queue.
  void allocate_by_rate(double T, double q) {
    const int32_t g_rate = gamma_for_rate(q);
    for (Batch& b : queue) {
      const double mean_u = b.u_sum / (double)b.req.size();
      if (T + time_of(b, g_rate) >= b.d_b) b.gamma = g_smallest;
      else if (mean_u > p.kappa) b.gamma = g_largest;
      else b.gamma = g_rate;
      T = T + time_of(b, b.gamma);
    }
  }

  // The dynamic program of Alg. 2.  State (b, l): l = 0 batch b skipped, l = 1..NG batch b runs with
  // gammas[l - 1].  util / clock hold the best accumulated utility of a state and the clock after it; a
  // state no predecessor can reach in time is marked unreachable.  The first feasible predecessor of a
  // state is always taken, a later one only when strictly better.
  double allocate_by_dp(double T) {
    const int32_t NB = (int32_t)queue.size(), W = NG + 1;
    const double NEG = -std::numeric_limits<double>::infinity();
    std::vector<double> util_prev(W, 0.0), clock_prev(W, T), util(W), clock(W);
    std::vector<int32_t> pred((size_t)NB * W, 0);
    std::vector<double> t_hat(NG), U_hat(NG);
    for (int32_t b = 0; b < NB; ++b) {
      const Batch& bt = queue[b];
      for (int32_t g = 0; g < NG; ++g) {
        t_hat[g] = time_of(bt, g);
        U_hat[g] = utility_of(bt, g);
      }
      for (int32_t l = 0; l < W; ++l) {
        bool reached = false;
        double best_u = NEG, best_c = std::numeric_limits<double>::infinity();
        int32_t best_p = 0;
        for (int32_t lp = 0; lp < W; ++lp) {
          if (util_prev[lp] == NEG) continue;
          double u, c;
          if (l == 0) {
            u = util_prev[lp];
            c = clock_prev[lp];
          } else {
            c = clock_prev[lp] + t_hat[l - 1];
            if (!(c < bt.d_b)) continue;
            u = util_prev[lp] + U_hat[l - 1];
          }
          if (!reached || u > best_u) {
            reached = true;
            best_u = u;
            best_c = c;
            best_p = lp;
          }
        }
        util[l] = best_u;
        clock[l] = best_c;
        pred[(size_t)b * W + l] = best_p;
      }
      util_prev.swap(util);
      clock_prev.swap(clock);
    }
    int32_t l = 0;
    for (int32_t i = 1; i < W; ++i)
      if (util_prev[i] > util_prev[l]) l = i;
    const double best = util_prev[l];
    for (int32_t b = NB - 1; b >= 0; --b) {
      queue[b].gamma = l == 0 ? OTAS_GAMMA_SKIP : l - 1;
      l = pred[(size_t)b * W + l];
    }
    return best;
  }
};

extern "C" {

int otas_sched_create(const otas_sched_params* params, int32_t n_gamma, const int32_t* gammas, int32_t n_tasks,
                      const double* latency, const double* accuracy, int32_t n_rate, const double* rate_max,
                      const int32_t* rate_gamma, otas_sched** out) {
  if (!params || !gammas || !latency || !accuracy || !out) return OTAS_EINVAL;
  if (n_gamma < 1 || n_tasks < 1 || n_rate < 0 || (n_rate > 0 && (!rate_max || !rate_gamma))) return OTAS_EINVAL;
  if (params->epsilon < 1 || params->beta < 0 || !(params->delta >= 0) || !(params->eta >= 0) || !(params->mu >= 0) ||
      std::isnan(params->kappa))
    return OTAS_EINVAL;
  for (int32_t i = 0; i < n_gamma; ++i)
    for (int32_t j = 0; j < i; ++j)
      if (gammas[i] == gammas[j]) return OTAS_EINVAL;
  for (int64_t i = 0; i < (int64_t)n_gamma * n_tasks; ++i)
    if (!(latency[i] > 0) || std::isnan(accuracy[i])) return OTAS_EINVAL;
  for (int32_t i = 0; i < n_rate; ++i) {
    if (rate_gamma[i] < 0 || rate_gamma[i] >= n_gamma || std::isnan(rate_max[i])) return OTAS_EINVAL;
    if (i > 0 && rate_max[i] < rate_max[i - 1]) return OTAS_EINVAL;
  }
  otas_sched* s = new (std::nothrow) otas_sched();
  if (!s) return OTAS_ENOMEM;
  try {
    s->p = *params;
    s->NG = n_gamma;
    s->NT = n_tasks;
    s->gammas.assign(gammas, gammas + n_gamma);
    s->latency.assign(latency, latency + (size_t)n_gamma * n_tasks);
    s->accuracy.assign(accuracy, accuracy + (size_t)n_gamma * n_tasks);
    if (n_rate > 0) {
      s->rate_max.assign(rate_max, rate_max + n_rate);
      s->rate_gamma.assign(rate_gamma, rate_gamma + n_rate);
    }
    s->g_smallest = (int32_t)(std::min_element(s->gammas.begin(), s->gammas.end()) - s->gammas.begin());
    s->g_largest = (int32_t)(std::max_element(s->gammas.begin(), s->gammas.end()) - s->gammas.begin());
  } catch (const std::bad_alloc&) {
    delete s;
    return OTAS_ENOMEM;
  }
  *out = s;
  return OTAS_OK;
}

void otas_sched_destroy(otas_sched* s) { delete s; }

int otas_sched_add_query(otas_sched* s, int64_t id, double s_r, double l_r, double u_r, int32_t task,
                         int32_t* batch) {
  if (!s || task < 0 || task >= s->NT || std::isnan(s_r) || std::isnan(l_r) || std::isnan(u_r)) return OTAS_EINVAL;
  const double d_r = s_r + l_r;
  const Request r{id, u_r, task};
  for (int32_t b = (int32_t)s->queue.size() - 1; b >= 0; --b) {
    Batch& bt = s->queue[b];
    if (bt.s_b + s->p.delta < s_r) break;                          // waited too long: stop looking
    if ((int32_t)bt.req.size() >= s->p.epsilon) continue;          // full
    if (std::fabs(bt.d_b - d_r) > s->p.eta) continue;              // deadlines too far apart
    if (std::fabs(bt.u_first - u_r) > s->p.mu) continue;           // utilities too far apart
    try {
      bt.req.push_back(r);
    } catch (const std::bad_alloc&) {
      return OTAS_ENOMEM;
    }
    bt.per_task[task] += 1;
    bt.s_b = std::min(bt.s_b, s_r);
    bt.d_b = std::min(bt.d_b, d_r);
    bt.u_sum += u_r;
    if (batch) *batch = b;
    return OTAS_OK;
  }
  try {
    Batch nb;
    nb.req.push_back(r);
    nb.per_task.assign(s->NT, 0);
    nb.per_task[task] = 1;
    nb.s_b = s_r;
    nb.d_b = d_r;
    nb.u_first = u_r;
    nb.u_sum = u_r;
    nb.gamma = OTAS_GAMMA_UNDECIDED;
    s->queue.push_back(std::move(nb));
  } catch (const std::bad_alloc&) {
    return OTAS_ENOMEM;
  }
  if (batch) *batch = (int32_t)s->queue.size() - 1;
  return OTAS_OK;
}

int otas_sched_allocate(otas_sched* s, double T, double q, int32_t initial_stage, double* planned_utility) {
  if (!s || std::isnan(T) || std::isnan(q)) return OTAS_EINVAL;
  if (planned_utility) *planned_utility = std::numeric_limits<double>::quiet_NaN();
  if (s->queue.empty()) return OTAS_OK;
  try {   // the sort's buffer and the tables are the only allocations; the gammas are written last
    std::stable_sort(s->queue.begin(), s->queue.end(), [](const Batch& a, const Batch& b) { return a.d_b < b.d_b; });
    if ((int32_t)s->queue.size() <= s->p.beta || initial_stage) {
      s->allocate_by_rate(T, q);
    } else {
      const double best = s->allocate_by_dp(T);
      if (planned_utility) *planned_utility = best;
    }
  } catch (const std::bad_alloc&) {
    return OTAS_ENOMEM;
  }
  return OTAS_OK;
}

int32_t otas_sched_num_batches(const otas_sched* s) { return s ? (int32_t)s->queue.size() : 0; }

int otas_sched_batch_info(const otas_sched* s, int32_t b, int32_t* size, double* s_b, double* d_b, double* u_b,
                          int32_t* gamma_index) {
  if (!s || b < 0 || b >= (int32_t)s->queue.size()) return OTAS_EINVAL;
  const Batch& bt = s->queue[b];
  if (size) *size = (int32_t)bt.req.size();
  if (s_b) *s_b = bt.s_b;
  if (d_b) *d_b = bt.d_b;
  if (u_b) *u_b = bt.u_first;
  if (gamma_index) *gamma_index = bt.gamma;
  return OTAS_OK;
}

int otas_sched_batch_queries(const otas_sched* s, int32_t b, int64_t* ids, int32_t* tasks, int32_t cap,
                             int32_t* n) {
  if (!s || b < 0 || b >= (int32_t)s->queue.size() || cap < 0) return OTAS_EINVAL;
  const Batch& bt = s->queue[b];
  const int32_t m = std::min<int32_t>(cap, (int32_t)bt.req.size());
  for (int32_t i = 0; i < m; ++i) {
    if (ids) ids[i] = bt.req[i].id;
    if (tasks) tasks[i] = bt.req[i].task;
  }
  if (n) *n = (int32_t)bt.req.size();
  return OTAS_OK;
}

int otas_sched_estimate(const otas_sched* s, int32_t b, int32_t gamma_index, double* t_hat, double* U_hat) {
  if (!s || b < 0 || b >= (int32_t)s->queue.size() || gamma_index < 0 || gamma_index >= s->NG) return OTAS_EINVAL;
  if (t_hat) *t_hat = s->time_of(s->queue[b], gamma_index);
  if (U_hat) *U_hat = s->utility_of(s->queue[b], gamma_index);
  return OTAS_OK;
}

int otas_sched_rate_table(int32_t n_gamma, const int32_t* gammas, int32_t n_tasks, const double* latency,
                          double* rate_max, int32_t* rate_gamma, int32_t* n_rate) {
  if (!gammas || !latency || !rate_max || !rate_gamma || !n_rate || n_gamma <= 0 || n_tasks <= 0) return OTAS_EINVAL;
  for (int32_t i = 0; i < n_tasks * n_gamma; ++i)
    if (!(latency[i] > 0.0)) return OTAS_EINVAL;
  // gamma indices from the largest gamma down (stable: equal gammas keep their list order)
  std::vector<int32_t> order(n_gamma);
  for (int32_t i = 0; i < n_gamma; ++i) order[i] = i;
  std::stable_sort(order.begin(), order.end(), [&](int32_t a, int32_t b) { return gammas[a] > gammas[b]; });
  int32_t rows = 0;
  for (int32_t k = 0; k + 1 < n_gamma; ++k) {   // the smallest gamma needs no row
    const int32_t gi = order[k];
    double sum = 0.0;
    for (int32_t t = 0; t < n_tasks; ++t) sum += latency[(size_t)t * n_gamma + gi];   // tasks in ascending order
    const double thr = 1.0 / (sum / (double)n_tasks);
    if (rows == 0 || thr > rate_max[rows - 1]) {
      rate_max[rows] = thr;
      rate_gamma[rows] = gi;
      ++rows;
    }
  }
  *n_rate = rows;
  return OTAS_OK;
}

int otas_sched_remove(otas_sched* s, int32_t b) {
  if (!s || b < 0 || b >= (int32_t)s->queue.size()) return OTAS_EINVAL;
  s->queue.erase(s->queue.begin() + b);
  return OTAS_OK;
}

}  // extern "C"
