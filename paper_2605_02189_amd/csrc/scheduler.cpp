// Prefetch-aware decode scheduler (PipeMax Sec. 3.3, App. A.4): host code only.
//
// The scheduler predicts the time of the step that is about to run (Eq. 2), converts it into the
// number of cached tokens the host link can deliver behind that step (Eq. 6) and picks the
// host-resident requests of the next batch to prefetch: shortest first while the budgets are still
// growing (warm-up), longest first plus count-adjusting exchanges once they have settled (steady;
// Alg. 1 and Alg. 2).  It drives a stage through the public calls of pipemax.h and mirrors the stage's
// bookkeeping so that a whole iteration can be planned before anything is enqueued.
#include <algorithm>
#include <cmath>
#include <cstdarg>
#include <cstdint>
#include <deque>
#include <numeric>
#include <vector>

#include "pipemax_sched.h"

#pragma STDC FP_CONTRACT OFF

namespace pmx {
void set_error(const char* fmt, ...);
}

#define SCHED_FAIL(code, ...)      \
  do {                             \
    ::pmx::set_error(__VA_ARGS__); \
    return (code);                 \
  } while (0)

namespace {

struct Request {
  int32_t len = 0;
  bool resident = false;
  int64_t since = -1;   // iteration whose prefetch brought the request in (-1: resident from the start)
};

struct Batch {
  bool declared = false;
  std::vector<Request> req;
};

// indices 0..n-1 ordered by length; descending or ascending, ties by index
std::vector<int32_t> order_by_len(const int32_t* len, int32_t n, bool descending) {
  std::vector<int32_t> o(n);
  std::iota(o.begin(), o.end(), 0);
  if (descending)
    std::sort(o.begin(), o.end(), [&](int32_t a, int32_t b) { return len[a] != len[b] ? len[a] > len[b] : a < b; });
  else
    std::sort(o.begin(), o.end(), [&](int32_t a, int32_t b) { return len[a] != len[b] ? len[a] < len[b] : a < b; });
  return o;
}

void fill_short_first(const int32_t* len, int32_t n, int64_t budget, std::vector<int32_t>& sel) {
  sel.clear();
  int64_t S = 0;
  for (int32_t r : order_by_len(len, n, false)) {
    if (S + len[r] > budget) break;   // ascending order: nothing later fits either
    sel.push_back(r);
    S += len[r];
  }
}

void fill_long_first(const int32_t* len, int32_t n, int64_t budget, std::vector<int32_t>& sel) {
  sel.clear();
  int64_t S = 0;
  for (int32_t r : order_by_len(len, n, true))
    if (S + len[r] <= budget) {
      sel.push_back(r);
      S += len[r];
    }
}

// first position p in u[from, end) (u ordered by descending length) with len[u[p]] <= limit
size_t first_not_longer(const std::vector<int32_t>& u, const int32_t* len, size_t from, int64_t limit) {
  size_t lo = from, hi = u.size();
  while (lo < hi) {
    const size_t mid = (lo + hi) / 2;
    if ((int64_t)len[u[mid]] <= limit) hi = mid;
    else lo = mid + 1;
  }
  return lo;
}

struct RefineModel {
  double alpha, beta, tol;
  int max_steps;
};

// Exchange pass of Alg. 2.  Every exchange keeps the total length within the budget and is applied
// only if it moves alpha*|P| + beta*S closer to the gap.
int refine_selection(const RefineModel& m, const int32_t* len, int32_t n, int64_t budget, double gap,
                     std::vector<int32_t>& sel) {
  std::vector<char> in(n, 0);
  for (int32_t r : sel) in[r] = 1;
  const std::vector<int32_t> desc = order_by_len(len, n, true);
  int applied_total = 0;
  for (int step = 0; step < m.max_steps; ++step) {
    int64_t S = 0;
    for (int32_t r : sel) S += len[r];
    const double mis = (m.alpha * (double)sel.size() + m.beta * (double)S) - gap;
    if (std::fabs(mis) <= m.tol) break;
    std::vector<int32_t> out_desc, in_desc;   // unselected / selected, longest first
    for (int32_t r : desc) (in[r] ? in_desc : out_desc).push_back(r);
    bool applied = false;
    if (mis < 0) {
      // too few requests for the time to fill: one long request against the best-fitting pair of shorter ones
      for (int32_t r : in_desc) {
        const int64_t cap = budget - (S - len[r]);
        const size_t p0 = first_not_longer(out_desc, len, 0, (int64_t)len[r] - 1);
        int64_t best = -1;
        int32_t bu = -1, bv = -1;
        for (size_t x = p0; x + 1 < out_desc.size(); ++x) {
          const int64_t lx = len[out_desc[x]];
          if (lx + len[out_desc[x + 1]] <= best) break;   // no later pair can be strictly larger
          const size_t y = first_not_longer(out_desc, len, x + 1, cap - lx);
          if (y >= out_desc.size()) continue;
          const int64_t tot = lx + len[out_desc[y]];
          if (tot > best) {
            best = tot;
            bu = out_desc[x];
            bv = out_desc[y];
          }
        }
        if (best < 0) continue;
        const int64_t S2 = S - len[r] + best;
        const double mis2 = (m.alpha * (double)(sel.size() + 1) + m.beta * (double)S2) - gap;
        if (std::fabs(mis2) < std::fabs(mis)) {
          sel.erase(std::find(sel.begin(), sel.end(), r));
          sel.push_back(bu);
          sel.push_back(bv);
          in[r] = 0;
          in[bu] = in[bv] = 1;
          applied = true;
          break;
        }
      }
    } else {
      // too many requests: two neighbouring short ones against the longest unselected one that fits
      std::vector<int32_t> asc = sel;
      std::sort(asc.begin(), asc.end(), [&](int32_t a, int32_t b) { return len[a] != len[b] ? len[a] < len[b] : a < b; });
      for (size_t q = 0; q + 1 < asc.size(); ++q) {
        const int32_t a = asc[q], b = asc[q + 1];
        const int64_t cap = budget - (S - len[a] - len[b]);
        const size_t p = first_not_longer(out_desc, len, 0, cap);
        if (p >= out_desc.size() || len[out_desc[p]] <= len[b]) continue;
        const int32_t u = out_desc[p];
        const int64_t S2 = S - len[a] - len[b] + len[u];
        const double mis2 = (m.alpha * (double)(sel.size() - 1) + m.beta * (double)S2) - gap;
        if (std::fabs(mis2) < std::fabs(mis)) {
          sel.erase(std::find(sel.begin(), sel.end(), a));
          sel.erase(std::find(sel.begin(), sel.end(), b));
          sel.push_back(u);
          in[a] = in[b] = 0;
          in[u] = 1;
          applied = true;
          break;
        }
      }
    }
    if (!applied) break;
    ++applied_total;
  }
  return applied_total;
}

int64_t pages_for(int64_t tokens, int32_t page_tokens) { return (tokens + page_tokens - 1) / page_tokens; }

}  // namespace

struct pipemax_sched {
  pipemax_sched_config_t cfg{};
  std::deque<int64_t> window;
  bool steady = false;
  std::vector<Batch> batch;
  int64_t gpu_free = 0;
  bool free_known = false;

  double predict(int64_t b, int64_t L) const { return cfg.alpha_s * (double)b + cfg.beta_s * (double)L + cfg.delta_s; }
  int64_t budget(double t_hat) const {
    if (cfg.static_budget_tokens > 0) return cfg.static_budget_tokens;
    return (int64_t)std::floor(cfg.link_tokens_per_s * t_hat);
  }
  bool observe(int64_t b) {
    window.push_back(b);
    if ((int)window.size() > cfg.window) window.pop_front();
    if (!steady && (int)window.size() == cfg.window) {
      int64_t lo = window.front(), hi = window.front(), sum = 0;
      for (int64_t v : window) {
        lo = std::min(lo, v);
        hi = std::max(hi, v);
        sum += v;
      }
      const double mean = (double)sum / (double)cfg.window;
      if (mean > 0 && (double)(hi - lo) / mean < cfg.steady_rel_range) steady = true;
    }
    return steady;
  }
};

namespace {

struct Plan {
  pipemax_sched_iter_t info{};
  std::vector<int32_t> exec, prefetch, evict;
};

// Alg. 1, one iteration, on the mirror.  On success the mirror has advanced.
int plan_iteration(pipemax_sched* s, int64_t t, Plan& P) {
  const int n = s->cfg.n_batches, pt = s->cfg.page_tokens;
  if (t < 0) SCHED_FAIL(PIPEMAX_ERR_ARG, "negative iteration");
  if (!s->free_known) SCHED_FAIL(PIPEMAX_ERR_STATE, "free GPU pages unknown: attach a stage or set them");
  const int i = (int)(t % n), j = (i + 1) % n, k = (i + n - 1) % n;
  for (int m : {i, j, k})
    if (!s->batch[m].declared) SCHED_FAIL(PIPEMAX_ERR_STATE, "batch %d is not declared", m);
  Batch& Bi = s->batch[i];
  P.exec.clear();
  P.prefetch.clear();
  P.evict.clear();
  int64_t L_exec = 0, grow = 0;
  for (int32_t q = 0; q < (int32_t)Bi.req.size(); ++q)
    if (Bi.req[q].resident) {
      P.exec.push_back(q);
      L_exec += Bi.req[q].len;
      grow += (Bi.req[q].len % pt == 0);
    }
  if (grow > s->gpu_free)
    SCHED_FAIL(PIPEMAX_ERR_STATE, "%lld new pages for the step, %lld free", (long long)grow, (long long)s->gpu_free);
  const double t_hat = s->predict((int64_t)P.exec.size(), L_exec);
  const int64_t budget = s->budget(t_hat);
  const bool steady = s->observe(budget);
  s->gpu_free -= grow;
  for (int32_t q : P.exec) Bi.req[q].len += 1;

  double gap = 0.0;
  int n_ex = 0;
  int64_t pf_tokens = 0;
  if (j != i) {
    Batch& Bj = s->batch[j];
    std::vector<int32_t> cand, cand_len;
    int64_t L_res = 0, n_res = 0, grow_res = 0;
    for (int32_t q = 0; q < (int32_t)Bj.req.size(); ++q) {
      if (Bj.req[q].resident) {
        ++n_res;
        L_res += Bj.req[q].len;
        grow_res += (Bj.req[q].len % pt == 0);
      } else {
        cand.push_back(q);
        cand_len.push_back(Bj.req[q].len);
      }
    }
    gap = t_hat - s->predict(n_res, L_res);
    std::vector<int32_t> pick;
    if (steady) {
      fill_long_first(cand_len.data(), (int32_t)cand.size(), budget, pick);
      const RefineModel m{s->cfg.alpha_s, s->cfg.beta_s, s->cfg.refine_tol_s, s->cfg.max_refine_steps};
      n_ex = refine_selection(m, cand_len.data(), (int32_t)cand.size(), budget, gap, pick);
    } else {
      fill_short_first(cand_len.data(), (int32_t)cand.size(), budget, pick);
    }
    // pages the prefetch takes plus the new pages of the step that will execute D_j
    auto need_of = [&](size_t count) {
      int64_t need = grow_res;
      for (size_t x = 0; x < count; ++x) {
        const int32_t len = cand_len[pick[x]];
        need += pages_for(len, pt) + (len % pt == 0);
      }
      return need;
    };
    int64_t need = need_of(pick.size());
    if (k != i && k != j && s->gpu_free < need) {
      Batch& Bk = s->batch[k];
      std::vector<int32_t> order;
      for (int32_t q = 0; q < (int32_t)Bk.req.size(); ++q)
        if (Bk.req[q].resident) order.push_back(q);
      std::stable_sort(order.begin(), order.end(),
                       [&](int32_t a, int32_t b) { return Bk.req[a].since < Bk.req[b].since; });
      for (int32_t q : order) {
        if (s->gpu_free >= need) break;
        s->gpu_free += pages_for(Bk.req[q].len, pt);
        Bk.req[q].resident = false;
        P.evict.push_back(q);
      }
    }
    size_t keep = pick.size();
    while (keep > 0 && s->gpu_free < need) need = need_of(--keep);
    if (s->gpu_free < need)
      SCHED_FAIL(PIPEMAX_ERR_STATE, "no room for the new pages of the next step (%lld needed, %lld free)",
                 (long long)need, (long long)s->gpu_free);
    for (size_t x = 0; x < keep; ++x) {
      Request& R = Bj.req[cand[pick[x]]];
      s->gpu_free -= pages_for(R.len, pt);
      R.resident = true;
      R.since = t;
      pf_tokens += R.len;
      P.prefetch.push_back(cand[pick[x]]);
    }
  }
  pipemax_sched_iter_t& o = P.info;
  o.exec_batch = i;
  o.n_exec = (int32_t)P.exec.size();
  o.prefetch_batch = j;
  o.n_prefetch = (int32_t)P.prefetch.size();
  o.evict_batch = k;
  o.n_evict = (int32_t)P.evict.size();
  o.steady = steady ? 1 : 0;
  o.n_exchanges = n_ex;
  o.budget_tokens = budget;
  o.prefetch_tokens = pf_tokens;
  o.gpu_pages_free = s->gpu_free;
  o.t_hat_s = t_hat;
  o.gap_s = gap;
  return PIPEMAX_OK;
}

void export_plan(const Plan& P, pipemax_sched_iter_t* out, int32_t* e, int32_t* p, int32_t* v) {
  if (out) *out = P.info;
  if (e) std::copy(P.exec.begin(), P.exec.end(), e);
  if (p) std::copy(P.prefetch.begin(), P.prefetch.end(), p);
  if (v) std::copy(P.evict.begin(), P.evict.end(), v);
}

int check_lens(const int32_t* len, int32_t n, const void* a, const void* b) {
  if (n < 0 || (n > 0 && !len) || !a || !b) SCHED_FAIL(PIPEMAX_ERR_ARG, "null argument or negative count");
  for (int32_t r = 0; r < n; ++r)
    if (len[r] < 0) SCHED_FAIL(PIPEMAX_ERR_ARG, "negative length at index %d", r);
  return PIPEMAX_OK;
}

}  // namespace

extern "C" {

int pipemax_sched_create(const pipemax_sched_config_t* cfg, pipemax_sched_t** out) {
  if (!cfg || !out) SCHED_FAIL(PIPEMAX_ERR_ARG, "null argument");
  *out = nullptr;
  const pipemax_sched_config_t& c = *cfg;
  if (c.window < 1 || c.max_refine_steps < 0 || c.n_batches < 1 || c.page_tokens < 1)
    SCHED_FAIL(PIPEMAX_ERR_ARG, "window, n_batches, page_tokens must be >= 1 and max_refine_steps >= 0");
  if (!(c.alpha_s >= 0) || !(c.beta_s >= 0) || !(c.delta_s >= 0) || !(c.link_tokens_per_s >= 0) ||
      !(c.steady_rel_range >= 0) || !(c.refine_tol_s >= 0) || c.static_budget_tokens < 0)
    SCHED_FAIL(PIPEMAX_ERR_ARG, "negative or NaN model parameter");
  pipemax_sched* s = new pipemax_sched();
  s->cfg = c;
  s->batch.resize(c.n_batches);
  *out = s;
  return PIPEMAX_OK;
}

int pipemax_sched_destroy(pipemax_sched_t* s) {
  if (!s) SCHED_FAIL(PIPEMAX_ERR_ARG, "null scheduler");
  delete s;
  return PIPEMAX_OK;
}

double pipemax_sched_predict(const pipemax_sched_t* s, int32_t b, int64_t total_len) {
  return s ? s->predict(b, total_len) : std::nan("");
}

int64_t pipemax_sched_budget(const pipemax_sched_t* s, double t_hat_s) { return s ? s->budget(t_hat_s) : -1; }

int pipemax_sched_observe(pipemax_sched_t* s, int64_t budget_tokens) {
  if (!s) SCHED_FAIL(PIPEMAX_ERR_ARG, "null scheduler");
  return s->observe(budget_tokens) ? 1 : 0;
}

int pipemax_sched_short_first_fill(const int32_t* len, int32_t n, int64_t budget, int32_t* sel, int32_t* n_sel) {
  int rc = check_lens(len, n, n > 0 ? (const void*)sel : (const void*)n_sel, n_sel);
  if (rc) return rc;
  std::vector<int32_t> v;
  fill_short_first(len, n, budget, v);
  std::copy(v.begin(), v.end(), sel);
  *n_sel = (int32_t)v.size();
  return PIPEMAX_OK;
}

int pipemax_sched_greedy_fill(const int32_t* len, int32_t n, int64_t budget, int32_t* sel, int32_t* n_sel) {
  int rc = check_lens(len, n, n > 0 ? (const void*)sel : (const void*)n_sel, n_sel);
  if (rc) return rc;
  std::vector<int32_t> v;
  fill_long_first(len, n, budget, v);
  std::copy(v.begin(), v.end(), sel);
  *n_sel = (int32_t)v.size();
  return PIPEMAX_OK;
}

int pipemax_sched_refine(const pipemax_sched_t* s, const int32_t* len, int32_t n, int64_t budget, double gap_s,
                         int32_t* sel, int32_t* n_sel, int32_t* n_exchanges) {
  if (!s) SCHED_FAIL(PIPEMAX_ERR_ARG, "null scheduler");
  int rc = check_lens(len, n, n > 0 ? (const void*)sel : (const void*)n_sel, n_sel);
  if (rc) return rc;
  if (*n_sel < 0 || *n_sel > n) SCHED_FAIL(PIPEMAX_ERR_ARG, "selection of %d out of %d requests", *n_sel, n);
  std::vector<int32_t> v(sel, sel + *n_sel);
  std::vector<char> seen(n, 0);
  int64_t S = 0;
  for (int32_t r : v) {
    if (r < 0 || r >= n || seen[r]) SCHED_FAIL(PIPEMAX_ERR_ARG, "selected index %d out of range or listed twice", r);
    seen[r] = 1;
    S += len[r];
  }
  if (S > budget) SCHED_FAIL(PIPEMAX_ERR_ARG, "the selection's %lld tokens exceed the budget", (long long)S);
  const RefineModel m{s->cfg.alpha_s, s->cfg.beta_s, s->cfg.refine_tol_s, s->cfg.max_refine_steps};
  const int ex = refine_selection(m, len, n, budget, gap_s, v);
  std::copy(v.begin(), v.end(), sel);
  *n_sel = (int32_t)v.size();
  if (n_exchanges) *n_exchanges = ex;
  return PIPEMAX_OK;
}

int pipemax_sched_partition(const int32_t* len, int32_t n, int32_t n_batches, int32_t* batch_of) {
  int rc = check_lens(len, n, n > 0 ? (const void*)batch_of : (const void*)&n, &n);
  if (rc) return rc;
  if (n_batches < 1) SCHED_FAIL(PIPEMAX_ERR_ARG, "n_batches must be >= 1");
  const std::vector<int32_t> desc = order_by_len(len, n, true);
  // serpentine deal: 0..n-1, n-1..0, 0..n-1, ...  Sizes differ by at most one and the long and the
  // short request of every double round meet in the same batch.
  for (int32_t pos = 0; pos < n; ++pos) {
    const int32_t round = pos / n_batches, k = pos % n_batches;
    batch_of[desc[pos]] = (round & 1) ? (n_batches - 1 - k) : k;
  }
  return PIPEMAX_OK;
}

int pipemax_sched_set_batch(pipemax_sched_t* s, int32_t mb, int32_t n, const int32_t* len, const int32_t* resident) {
  if (!s) SCHED_FAIL(PIPEMAX_ERR_ARG, "null scheduler");
  if (mb < 0 || mb >= s->cfg.n_batches) SCHED_FAIL(PIPEMAX_ERR_ARG, "batch %d out of range", mb);
  int rc = check_lens(len, n, n > 0 ? (const void*)resident : (const void*)s, s);
  if (rc) return rc;
  Batch& B = s->batch[mb];
  B.req.assign(n, Request());
  for (int32_t r = 0; r < n; ++r) {
    B.req[r].len = len[r];
    B.req[r].resident = resident[r] != 0;
  }
  B.declared = true;
  return PIPEMAX_OK;
}

int pipemax_sched_set_gpu_pages_free(pipemax_sched_t* s, int64_t pages) {
  if (!s || pages < 0) SCHED_FAIL(PIPEMAX_ERR_ARG, "null scheduler or negative page count");
  s->gpu_free = pages;
  s->free_known = true;
  return PIPEMAX_OK;
}

int pipemax_sched_attach(pipemax_sched_t* s, pipemax_stage_t* stage) {
  if (!s || !stage) SCHED_FAIL(PIPEMAX_ERR_ARG, "null argument");
  pipemax_config_t sc;
  int rc = pipemax_get_config(stage, &sc);
  if (rc) return rc;
  if (sc.n_microbatches != s->cfg.n_batches || sc.page_tokens != s->cfg.page_tokens)
    SCHED_FAIL(PIPEMAX_ERR_ARG, "the stage has %d micro-batches of %d-token pages, the scheduler %d of %d",
               sc.n_microbatches, sc.page_tokens, s->cfg.n_batches, s->cfg.page_tokens);
  for (int mb = 0; mb < sc.n_microbatches; ++mb) {
    int32_t b = 0;
    if ((rc = pipemax_mb_size(stage, mb, &b))) return rc;
    if (b == 0) SCHED_FAIL(PIPEMAX_ERR_STATE, "micro-batch %d of the stage is not defined", mb);
    std::vector<int32_t> len(b), res(b);
    if ((rc = pipemax_get_ctx_lens(stage, mb, len.data()))) return rc;
    if ((rc = pipemax_get_residency(stage, mb, res.data()))) return rc;
    if ((rc = pipemax_sched_set_batch(s, mb, b, len.data(), res.data()))) return rc;
  }
  pipemax_stats_t stt;
  if ((rc = pipemax_get_stats(stage, &stt))) return rc;
  return pipemax_sched_set_gpu_pages_free(s, stt.gpu_pages_free);
}

int pipemax_sched_plan(pipemax_sched_t* s, int64_t t, pipemax_sched_iter_t* out, int32_t* exec_ids,
                       int32_t* prefetch_ids, int32_t* evict_ids) {
  if (!s) SCHED_FAIL(PIPEMAX_ERR_ARG, "null scheduler");
  const pipemax_sched saved = *s;
  Plan P;
  int rc = plan_iteration(s, t, P);
  if (rc) {
    *s = saved;
    return rc;
  }
  export_plan(P, out, exec_ids, prefetch_ids, evict_ids);
  return PIPEMAX_OK;
}

int pipemax_sched_iterate(pipemax_sched_t* s, pipemax_stage_t* stage, int64_t t, const void* hidden_in,
                          void* hidden_out, void* hip_stream, pipemax_sched_iter_t* out, int32_t* exec_ids,
                          int32_t* prefetch_ids, int32_t* evict_ids) {
  if (!s || !stage) SCHED_FAIL(PIPEMAX_ERR_ARG, "null argument");
  const pipemax_sched saved = *s;
  Plan P;
  int rc = plan_iteration(s, t, P);
  if (rc) {
    *s = saved;
    return rc;
  }
  // The transfers first: neither call blocks (the stage's prefetch worker waits for the last reader of the released
  // pages), and the copies then start the moment the previous step ends instead of after the host has spent its
  // 0.2-0.3 ms enqueuing this one -- the copy has exactly one step to finish in (measured on a kernel / copy trace:
  // issued after the step, the copies of an iteration ended 0.1-0.2 ms after the step they were meant to hide behind).
  if (!P.evict.empty())
    rc = pipemax_evict_kv(stage, P.info.evict_batch, P.evict.data(), (int)P.evict.size());
  if (!rc && !P.prefetch.empty())
    rc = pipemax_prefetch_kv(stage, P.info.prefetch_batch, P.prefetch.data(), (int)P.prefetch.size());
  if (!rc)
    rc = pipemax_decode_step_seqs(stage, P.info.exec_batch, P.exec.data(), (int)P.exec.size(), hidden_in, hidden_out,
                                  hip_stream);
  if (rc) {
    *s = saved;
    return rc;
  }
  pipemax_stats_t stt;
  if ((rc = pipemax_get_stats(stage, &stt))) return rc;
  if ((int64_t)stt.gpu_pages_free != s->gpu_free)
    SCHED_FAIL(PIPEMAX_ERR_STATE, "the stage has %d free GPU pages, the scheduler's mirror %lld", stt.gpu_pages_free,
               (long long)s->gpu_free);
  export_plan(P, out, exec_ids, prefetch_ids, evict_ids);
  return PIPEMAX_OK;
}

}  // extern "C"
