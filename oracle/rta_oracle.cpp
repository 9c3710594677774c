/*
 * CPU oracle for the GCAPS response-time analyses.  TEST INFRASTRUCTURE ONLY:
 * see rta_oracle.h.  Plain C++17, int64 arithmetic, one thread per call of
 * oracle_rta_taskset, no blocking, fusion or reordering of the paper's sums.
 *
 * Notation follows Sec. 3 and Sec. 5: C_i, G^m_i, G^e_i, G_i, T_i, D_i,
 * eta^g_i, hp(tau_i), hpp(tau_i), theta, epsilon, L, J^c_h, J^g_h.
 */
#include "rta_oracle.h"

#include <algorithm>
#include <limits>
#include <numeric>
#include <thread>
#include <vector>

namespace {

using i64 = int64_t;

constexpr i64 kSat = std::numeric_limits<i64>::max();

/* Products and sums of non-negative quantities.  A result that does not fit in
 * int64 is replaced by the largest int64; such a value is larger than any
 * deadline (deadlines are < 2^32), so the verdict "bound exceeds D_i" is the
 * same as with unbounded integers. */
i64 mul(i64 a, i64 b) {
  i64 r;
  return __builtin_mul_overflow(a, b, &r) ? kSat : r;
}
i64 add(i64 a, i64 b) {
  i64 r;
  return __builtin_add_overflow(a, b, &r) ? kSat : r;
}

/* ceil(a / b) for a >= 0, b >= 1 */
i64 ceil_div(i64 a, i64 b) { return (a + b - 1) / b; }

struct Task {
  i64 C;    /* C_i: sum of CPU segments */
  i64 Gm;   /* G^m_i = sum_j G^m_{i,j} */
  i64 Ge;   /* G^e_i = sum_j G^e_{i,j} */
  i64 G;    /* G_i := G^m_i + G^e_i (upper end of G_i <= G^m_i + G^e_i, Sec. 3) */
  i64 T, D;
  i64 eta;  /* eta^g_i */
  int core;
  std::vector<i64> ge_seg; /* G^e_{i,j}, j < eta^g_i */
  i64 R;    /* response-time bound once known */
  bool gpu() const { return eta > 0; }
};

struct Params {
  i64 theta, eps, L;
};

/* Eq. 3: delay of one pure GPU segment of length ge against nu other TSGs. */
i64 interleave(const Params &p, i64 nu, i64 ge) {
  return mul(mul(p.L + p.theta, nu), ceil_div(ge, p.L));
}

/* sum over the GPU segments of task x of Eq. 3 with nu interleaving TSGs */
i64 interleave_sum(const Params &p, i64 nu, const Task &x) {
  i64 s = 0;
  for (i64 ge : x.ge_seg) s = add(s, interleave(p, nu, ge));
  return s;
}

/* Task-model checks (Sec. 3: T >= 1, 1 <= D <= T, eta^g <= S, L >= 1), then the tasks in
 * decreasing CPU priority (equal priorities keep caller order): order[k] = caller index of
 * the task of rank k. */
int read_taskset(uint32_t n_tasks, uint32_t max_gseg, uint32_t slice_us, const uint32_t *cpu_us,
                 const uint32_t *period_us, const uint32_t *deadline_us, const int32_t *prio,
                 const uint8_t *core, const uint8_t *n_gseg, const uint32_t *gm_us,
                 const uint32_t *ge_us, std::vector<uint32_t> &order, std::vector<Task> &tau) {
  if (slice_us == 0) return ORACLE_ETASK;
  for (uint32_t i = 0; i < n_tasks; ++i) {
    if (period_us[i] == 0 || deadline_us[i] == 0 || deadline_us[i] > period_us[i]) return ORACLE_ETASK;
    if (n_gseg[i] > max_gseg) return ORACLE_ETASK;
  }
  order.resize(n_tasks);
  std::iota(order.begin(), order.end(), 0u);
  std::stable_sort(order.begin(), order.end(), [&](uint32_t a, uint32_t b) { return prio[a] > prio[b]; });
  tau.assign(n_tasks, Task());
  for (uint32_t k = 0; k < n_tasks; ++k) {
    uint32_t i = order[k];
    Task &t = tau[k];
    t.C = cpu_us[i];
    t.T = period_us[i];
    t.D = deadline_us[i];
    t.eta = n_gseg[i];
    t.core = core[i];
    t.Gm = t.Ge = 0;
    for (uint32_t j = 0; j < n_gseg[i]; ++j) {
      t.Gm += gm_us[(size_t)i * max_gseg + j];
      t.Ge += ge_us[(size_t)i * max_gseg + j];
      t.ge_seg.push_back(ge_us[(size_t)i * max_gseg + j]);
    }
    t.G = t.Gm + t.Ge;
    t.R = 0;
  }
  return ORACLE_OK;
}

bool valid_pointers(uint32_t n_tasks, uint32_t max_gseg, const void *cpu_us, const void *period_us,
                    const void *deadline_us, const void *prio, const void *core, const void *n_gseg,
                    const void *gm_us, const void *ge_us) {
  if (n_tasks == 0 || n_tasks > 255 || max_gseg > 255) return false;
  if (!cpu_us || !period_us || !deadline_us || !prio || !core || !n_gseg) return false;
  return max_gseg == 0 || (gm_us && ge_us);
}

struct Analysis {
  const std::vector<Task> &tau; /* priority order: index 0 is the highest priority */
  const Params &p;
  int policy, wait_mode;
  uint32_t options;
  uint64_t terms = 0;

  bool same_core(size_t h, size_t i) const { return tau[h].core == tau[i].core; }
  /* hp(tau_i) = {h < i}; hpp(tau_i) = {h < i : same core} (Lemma 4, Lemma 10) */

  /* starred demands of Sec. 5.3 */
  i64 Ge_star(const Task &t) const { return add(t.Ge, mul(2 * p.eps, t.eta)); }
  i64 Gm_star(const Task &t) const { return add(t.Gm, mul(2 * p.eps, t.eta)); }
  /* jitters of Lemma 7 and Lemma 10.  R_h >= C_h + G_h for a task that met its deadline; where
   * D_h stands in for an unknown R_h (continue-after-miss) a jitter is not taken below zero */
  i64 Jc(const Task &h) const { return std::max<i64>(0, h.R - (h.C + h.Gm)); }
  i64 Jg(const Task &h) const { return std::max<i64>(0, h.R - h.Ge); }

  i64 term(i64 window, i64 period, i64 cost) {
    ++terms;
    return mul(ceil_div(window, period), cost);
  }

  /* number of GPU-using tasks in the whole taskset */
  i64 n_gpu_tasks() const {
    i64 c = 0;
    for (const Task &t : tau) c += t.gpu();
    return c;
  }

  /* ---- R-independent part of R_i ---- */
  i64 base(size_t i) const {
    const Task &t = tau[i];
    i64 b = add(t.C, t.G); /* Eq. 1 */
    if (policy == ORACLE_POLICY_RR) {
      /* Lemma 1: I^ie_i against every other GPU-using task; Lemmas 2, 3: I^dp = B^C = 0 */
      i64 nu = n_gpu_tasks() - (t.gpu() ? 1 : 0);
      b = add(b, interleave_sum(p, nu, t));
    } else {
      /* Sec. 5.3: 2*eps per own GPU segment; Lemma 8: B^C_i = (eta+1)*eps; Lemma 9: I^ie = 0 */
      b = add(b, mul(2 * p.eps, t.eta));
      b = add(b, mul(t.eta + 1, p.eps));
    }
    return b;
  }

  /* ---- right-hand side of the recurrence for task i at window R ---- */
  i64 rr_busy(size_t i, i64 R) {
    i64 s = base(i);
    /* Lemma 5: P^C_i */
    for (size_t h = 0; h < i; ++h)
      if (same_core(h, i)) s = add(s, term(R, tau[h].T, tau[h].C + tau[h].Gm));
    /* Lemma 4: I^id_i.  Interleaving set: GPU-using tasks outside hpp(tau_i), plus tau_h. */
    i64 nu = 1;
    for (size_t k = 0; k < tau.size(); ++k) {
      bool in_hpp = k < i && same_core(k, i);
      if (!in_hpp && tau[k].gpu()) ++nu;
    }
    for (size_t h = 0; h < i; ++h)
      if (same_core(h, i) && tau[h].gpu()) s = add(s, term(R, tau[h].T, interleave_sum(p, nu, tau[h])));
    return s;
  }

  i64 rr_suspend(size_t i, i64 R) {
    i64 s = base(i); /* Lemma 6: I^id = 0 */
    /* Lemma 7: P^C_i with jitter J^c_h for self-suspending (GPU-using) tau_h */
    for (size_t h = 0; h < i; ++h)
      if (same_core(h, i)) {
        i64 J = tau[h].gpu() ? Jc(tau[h]) : 0;
        s = add(s, term(R + J, tau[h].T, tau[h].C + tau[h].Gm));
      }
    return s;
  }

  i64 gcaps_busy(size_t i, i64 R) {
    i64 s = base(i);
    /* Lemma 12: P^C_i */
    for (size_t h = 0; h < i; ++h)
      if (same_core(h, i)) s = add(s, term(R, tau[h].T, tau[h].C + tau[h].Gm));
    /* Lemma 10, first sum: busy-waiting same-core tau_h holds the CPU for G^{e*}_h.
     * Applied to every tau_i unless the literal guard eta^g_i > 0 is requested. */
    bool first_sum = tau[i].gpu() || !(options & ORACLE_OPT_LITERAL_LEMMA10);
    if (first_sum)
      for (size_t h = 0; h < i; ++h)
        if (same_core(h, i) && tau[h].gpu()) s = add(s, term(R, tau[h].T, Ge_star(tau[h])));
    /* Lemma 10, second sum (eta^g_i > 0) and Lemma 11 (eta^g_i = 0): the same expression */
    for (size_t h = 0; h < i; ++h)
      if (!same_core(h, i) && tau[h].gpu()) s = add(s, term(R + Jg(tau[h]), tau[h].T, Ge_star(tau[h])));
    return s;
  }

  i64 gcaps_suspend(size_t i, i64 R) {
    i64 s = base(i); /* Lemma 14: I^id = 0 */
    /* Lemma 15: P^C_i */
    for (size_t h = 0; h < i; ++h)
      if (same_core(h, i) && !tau[h].gpu()) s = add(s, term(R, tau[h].T, tau[h].C));
    for (size_t h = 0; h < i; ++h)
      if (same_core(h, i) && tau[h].gpu())
        s = add(s, term(R + Jc(tau[h]), tau[h].T, add(tau[h].C, Gm_star(tau[h]))));
    /* Lemma 13: I^dp_i, only for GPU-using tau_i */
    if (tau[i].gpu()) {
      for (size_t h = 0; h < i; ++h)
        if (same_core(h, i) && tau[h].gpu()) s = add(s, term(R + Jg(tau[h]), tau[h].T, tau[h].Ge));
      for (size_t h = 0; h < i; ++h)
        if (!same_core(h, i) && tau[h].gpu()) s = add(s, term(R + Jg(tau[h]), tau[h].T, Ge_star(tau[h])));
    }
    return s;
  }

  i64 rhs(size_t i, i64 R) {
    if (policy == ORACLE_POLICY_RR) return wait_mode == ORACLE_WAIT_BUSY ? rr_busy(i, R) : rr_suspend(i, R);
    return wait_mode == ORACLE_WAIT_BUSY ? gcaps_busy(i, R) : gcaps_suspend(i, R);
  }
};

/*
 * Sec. 5.4: the GCAPS analysis of Sec. 5.3 when GPU segments have priorities of their own.
 *  - hpp(tau_i) keeps its meaning (higher CPU priority, same core): an admissible GPU
 *    priority order agrees with the CPU priority order among the tasks of one core;
 *  - hp(tau_i) in the sums over tasks of OTHER cores (second sums of Lemmas 10 and 13,
 *    Lemma 11) is the set of tasks with a higher GPU-segment priority, `higher_g`;
 *  - every release jitter uses D_h in place of R_h.
 * With that, the bound of tau_i depends on the other tasks only through the SET higher_g,
 * which is what Audsley's assignment needs.  tau is in decreasing CPU priority.
 */
struct GprioAnalysis {
  const std::vector<Task> &tau;
  const Params &p;
  int wait_mode;
  uint32_t options;
  uint64_t terms = 0;

  bool on_core_of(size_t i, size_t h) const { return tau[h].core == tau[i].core; }
  bool uses_gpu(size_t h) const { return tau[h].eta > 0; }
  i64 updates(size_t h) const { return mul(2 * p.eps, tau[h].eta); } /* 2*eps per GPU segment, Sec. 5.3 */
  i64 ge_star(size_t h) const { return add(tau[h].Ge, updates(h)); }
  i64 gm_star(size_t h) const { return add(tau[h].Gm, updates(h)); }
  /* Lemma 7's J^c_h and Lemma 10's J^g_h with D_h for R_h; not below zero (only a task whose own
   * demand exceeds its deadline gets there, and the search settles such tasksets beforehand) */
  i64 jitter_c(size_t h) const { return std::max<i64>(0, tau[h].D - (tau[h].C + tau[h].Gm)); }
  i64 jitter_g(size_t h) const { return std::max<i64>(0, tau[h].D - tau[h].Ge); }

  i64 arrivals_times(i64 window, size_t h, i64 cost) {
    ++terms;
    return mul(ceil_div(window, tau[h].T), cost);
  }

  /* C_i + G_i, the two runlist updates per own GPU segment (Sec. 5.3), B^C_i (Lemma 8) */
  i64 base(size_t i) const {
    return add(add(add(tau[i].C, tau[i].G), updates(i)), mul(tau[i].eta + 1, p.eps));
  }

  i64 rhs(size_t i, i64 R, const std::vector<char> &higher_g) {
    i64 s = base(i);
    const size_t n = tau.size();
    if (wait_mode == ORACLE_WAIT_BUSY) {
      /* Lemma 12 */
      for (size_t h = 0; h < i; ++h)
        if (on_core_of(i, h)) s = add(s, arrivals_times(R, h, tau[h].C + tau[h].Gm));
      /* Lemma 10, first sum (for every tau_i unless the literal guard is asked for) */
      if (uses_gpu(i) || !(options & ORACLE_OPT_LITERAL_LEMMA10))
        for (size_t h = 0; h < i; ++h)
          if (on_core_of(i, h) && uses_gpu(h)) s = add(s, arrivals_times(R, h, ge_star(h)));
      /* Lemma 10, second sum (eta^g_i > 0); Lemma 11 (eta^g_i = 0) */
      for (size_t h = 0; h < n; ++h)
        if (higher_g[h] && !on_core_of(i, h) && uses_gpu(h))
          s = add(s, arrivals_times(R + jitter_g(h), h, ge_star(h)));
    } else {
      /* Lemma 15 */
      for (size_t h = 0; h < i; ++h)
        if (on_core_of(i, h) && !uses_gpu(h)) s = add(s, arrivals_times(R, h, tau[h].C));
      for (size_t h = 0; h < i; ++h)
        if (on_core_of(i, h) && uses_gpu(h))
          s = add(s, arrivals_times(R + jitter_c(h), h, add(tau[h].C, gm_star(h))));
      /* Lemma 13 */
      if (uses_gpu(i)) {
        for (size_t h = 0; h < i; ++h)
          if (on_core_of(i, h) && uses_gpu(h)) s = add(s, arrivals_times(R + jitter_g(h), h, tau[h].Ge));
        for (size_t h = 0; h < n; ++h)
          if (higher_g[h] && !on_core_of(i, h) && uses_gpu(h))
            s = add(s, arrivals_times(R + jitter_g(h), h, ge_star(h)));
      }
    }
    return s;
  }

  /* least fixed point from base(i); false when the bound exceeds D_i */
  bool solve(size_t i, const std::vector<char> &higher_g, i64 *out) {
    i64 R = base(i);
    if (R > tau[i].D) return false;
    for (;;) {
      i64 next = rhs(i, R, higher_g);
      if (next > tau[i].D) return false;
      if (next == R) break;
      R = next;
    }
    *out = R;
    return true;
  }
};

bool valid_selectors(int policy, int wait_mode) {
  return (policy == ORACLE_POLICY_GCAPS || policy == ORACLE_POLICY_RR) &&
         (wait_mode == ORACLE_WAIT_BUSY || wait_mode == ORACLE_WAIT_SUSPEND);
}

}  // namespace

extern "C" int oracle_rta_taskset(uint32_t n_tasks, uint32_t max_gseg, uint32_t theta_us,
                                  uint32_t eps_us, uint32_t slice_us, const uint32_t *cpu_us,
                                  const uint32_t *period_us, const uint32_t *deadline_us,
                                  const int32_t *prio, const uint8_t *core, const uint8_t *n_gseg,
                                  const uint32_t *gm_us, const uint32_t *ge_us, int policy,
                                  int wait_mode, uint32_t options, int64_t *resp, uint8_t *sched,
                                  uint64_t *terms) {
  if (!valid_pointers(n_tasks, max_gseg, cpu_us, period_us, deadline_us, prio, core, n_gseg, gm_us, ge_us) ||
      !resp || !sched)
    return ORACLE_EINVAL;
  if (!valid_selectors(policy, wait_mode)) return ORACLE_EINVAL;

  std::vector<uint32_t> order;
  std::vector<Task> tau;
  int rc = read_taskset(n_tasks, max_gseg, slice_us, cpu_us, period_us, deadline_us, prio, core, n_gseg,
                        gm_us, ge_us, order, tau);
  if (rc != ORACLE_OK) return rc;
  Params p{(i64)theta_us, (i64)eps_us, (i64)slice_us};

  Analysis a{tau, p, policy, wait_mode, options};
  bool missed = false;
  for (uint32_t k = 0; k < n_tasks; ++k) {
    uint32_t i = order[k];
    if (missed && !(options & ORACLE_OPT_CONTINUE_AFTER_MISS)) {
      resp[i] = ORACLE_RESP_NOT_ANALYSED;
      continue;
    }
    /* least fixed point of R = rhs(R), started at the R-independent part */
    i64 R = a.base(k);
    bool ok = R <= tau[k].D;
    while (ok) {
      i64 next = a.rhs(k, R);
      if (next > tau[k].D) {
        ok = false;
      } else if (next == R) {
        break;
      } else {
        R = next;
      }
    }
    if (ok) {
      tau[k].R = R;
      resp[i] = R;
    } else {
      missed = true;
      resp[i] = ORACLE_RESP_MISS;
      /* the response time of tau_k is unknown from here on: the jitters of the tasks below take
       * D_k in its place (proof of Lemma 10) */
      tau[k].R = tau[k].D;
    }
  }
  *sched = missed ? 0 : 1;
  if (terms) *terms = a.terms;
  return ORACLE_OK;
}

extern "C" int oracle_rta_batch(uint32_t n_tasksets, uint32_t n_tasks, uint32_t max_gseg,
                                const uint32_t *theta_us, const uint32_t *eps_us,
                                const uint32_t *slice_us, const uint32_t *cpu_us,
                                const uint32_t *period_us, const uint32_t *deadline_us,
                                const int32_t *prio, const uint8_t *core, const uint8_t *n_gseg,
                                const uint32_t *gm_us, const uint32_t *ge_us, int policy_mask,
                                int wait_mode, uint32_t options, int threads, int64_t *resp,
                                uint8_t *sched, uint64_t *terms_total, uint32_t *first_bad) {
  if (n_tasksets == 0 || !theta_us || !eps_us || !slice_us || !resp || !sched) return ORACLE_EINVAL;
  if (policy_mask < 1 || policy_mask > 3) return ORACLE_EINVAL;
  std::vector<int> policies;
  if (policy_mask & ORACLE_POLICY_GCAPS) policies.push_back(ORACLE_POLICY_GCAPS);
  if (policy_mask & ORACLE_POLICY_RR) policies.push_back(ORACLE_POLICY_RR);
  if (threads < 1) threads = 1;
  if ((uint32_t)threads > n_tasksets) threads = (int)n_tasksets;

  std::vector<int> rc(threads, ORACLE_OK);
  std::vector<uint32_t> bad(threads, 0xffffffffu);
  std::vector<uint64_t> terms(threads, 0);

  auto work = [&](int w) {
    uint32_t lo = (uint32_t)((uint64_t)n_tasksets * w / threads);
    uint32_t hi = (uint32_t)((uint64_t)n_tasksets * (w + 1) / threads);
    for (uint32_t s = lo; s < hi; ++s) {
      size_t to = (size_t)s * n_tasks;
      size_t so = to * max_gseg;
      for (size_t p = 0; p < policies.size(); ++p) {
        uint64_t t = 0;
        int r = oracle_rta_taskset(n_tasks, max_gseg, theta_us[s], eps_us[s], slice_us[s],
                                   cpu_us + to, period_us + to, deadline_us + to, prio + to,
                                   core + to, n_gseg + to, gm_us ? gm_us + so : nullptr,
                                   ge_us ? ge_us + so : nullptr, policies[p], wait_mode, options,
                                   resp + (p * n_tasksets + s) * (size_t)n_tasks,
                                   sched + p * n_tasksets + s, &t);
        if (r != ORACLE_OK) {
          rc[w] = r;
          bad[w] = s;
          return;
        }
        terms[w] += t;
      }
    }
  };

  if (threads == 1) {
    work(0);
  } else {
    std::vector<std::thread> pool;
    for (int w = 0; w < threads; ++w) pool.emplace_back(work, w);
    for (auto &th : pool) th.join();
  }
  uint64_t total = 0;
  for (int w = 0; w < threads; ++w) {
    total += terms[w];
    if (rc[w] != ORACLE_OK) {
      if (first_bad) *first_bad = bad[w];
      return rc[w];
    }
  }
  if (terms_total) *terms_total = total;
  return ORACLE_OK;
}

extern "C" int oracle_gprio_rta_taskset(uint32_t n_tasks, uint32_t max_gseg, uint32_t eps_us,
                                        const uint32_t *cpu_us, const uint32_t *period_us,
                                        const uint32_t *deadline_us, const int32_t *prio,
                                        const uint8_t *core, const uint8_t *n_gseg,
                                        const uint32_t *gm_us, const uint32_t *ge_us,
                                        const int32_t *gprio, int wait_mode, uint32_t options,
                                        int64_t *resp, uint8_t *sched, uint64_t *terms) {
  if (!valid_pointers(n_tasks, max_gseg, cpu_us, period_us, deadline_us, prio, core, n_gseg, gm_us, ge_us) ||
      !gprio || !resp || !sched)
    return ORACLE_EINVAL;
  if (wait_mode != ORACLE_WAIT_BUSY && wait_mode != ORACLE_WAIT_SUSPEND) return ORACLE_EINVAL;
  std::vector<uint32_t> order;
  std::vector<Task> tau;
  int rc = read_taskset(n_tasks, max_gseg, 1, cpu_us, period_us, deadline_us, prio, core, n_gseg, gm_us,
                        ge_us, order, tau);
  if (rc != ORACLE_OK) return rc;
  Params p{0, (i64)eps_us, 1};

  /* tau_a above tau_b in GPU priority; equal values fall back to the CPU priority order */
  auto above = [&](size_t a, size_t b) {
    return gprio[order[a]] != gprio[order[b]] ? gprio[order[a]] > gprio[order[b]] : a < b;
  };
  /* Sec. 4.3: among the tasks of one core the two orders must agree */
  for (size_t a = 0; a < n_tasks; ++a)
    for (size_t b = a + 1; b < n_tasks; ++b)
      if (tau[a].core == tau[b].core && !above(a, b)) return ORACLE_EORDER;

  GprioAnalysis g{tau, p, wait_mode, options};
  bool all = true;
  for (size_t k = 0; k < n_tasks; ++k) {
    std::vector<char> higher_g(n_tasks, 0);
    for (size_t h = 0; h < n_tasks; ++h) higher_g[h] = h != k && above(h, k);
    i64 R;
    if (g.solve(k, higher_g, &R)) {
      resp[order[k]] = R;
    } else {
      resp[order[k]] = ORACLE_RESP_MISS; /* tasks do not depend on each other's R here: all are analysed */
      all = false;
    }
  }
  *sched = all ? 1 : 0;
  if (terms) *terms = g.terms;
  return ORACLE_OK;
}

extern "C" int oracle_gprio_assign_taskset(uint32_t n_tasks, uint32_t max_gseg, uint32_t eps_us,
                                           const uint32_t *cpu_us, const uint32_t *period_us,
                                           const uint32_t *deadline_us, const int32_t *prio,
                                           const uint8_t *core, const uint8_t *n_gseg,
                                           const uint32_t *gm_us, const uint32_t *ge_us, int wait_mode,
                                           uint32_t options, int32_t *gprio, int64_t *resp,
                                           uint8_t *sched, uint64_t *terms) {
  if (!valid_pointers(n_tasks, max_gseg, cpu_us, period_us, deadline_us, prio, core, n_gseg, gm_us, ge_us) ||
      !gprio || !resp || !sched)
    return ORACLE_EINVAL;
  if (wait_mode != ORACLE_WAIT_BUSY && wait_mode != ORACLE_WAIT_SUSPEND) return ORACLE_EINVAL;
  std::vector<uint32_t> order;
  std::vector<Task> tau;
  int rc = read_taskset(n_tasks, max_gseg, 1, cpu_us, period_us, deadline_us, prio, core, n_gseg, gm_us,
                        ge_us, order, tau);
  if (rc != ORACLE_OK) return rc;
  Params p{0, (i64)eps_us, 1};
  GprioAnalysis g{tau, p, wait_mode, options};

  std::vector<char> unassigned(n_tasks, 1);
  std::vector<int32_t> level_of(n_tasks, 0);
  std::vector<i64> R_of(n_tasks, 0);
  bool ok = true;
  /* a task whose own demand exceeds its deadline passes at no level */
  for (size_t k = 0; k < n_tasks; ++k) ok = ok && g.base(k) <= tau[k].D;

  /* Sec. 4.3, Audsley's scheme: GPU priority levels from the lowest (1) to the highest (n) */
  for (uint32_t level = 1; ok && level <= n_tasks; ++level) {
    bool placed = false;
    /* candidates from the lowest to the highest CPU priority */
    for (size_t k = n_tasks; k-- > 0 && !placed;) {
      if (!unassigned[k]) continue;
      /* tau_k would end up below every task still unassigned: infeasible if one of them is a
       * lower-CPU-priority task of the same core */
      bool feasible = true;
      for (size_t m = k + 1; m < n_tasks; ++m)
        if (unassigned[m] && tau[m].core == tau[k].core) feasible = false;
      if (!feasible) continue;
      std::vector<char> higher_g(unassigned);
      higher_g[k] = 0;
      i64 R;
      if (g.solve(k, higher_g, &R)) {
        unassigned[k] = 0;
        level_of[k] = (int32_t)level;
        R_of[k] = R;
        placed = true;
      }
    }
    ok = placed;
  }
  for (size_t k = 0; k < n_tasks; ++k) {
    gprio[order[k]] = ok ? level_of[k] : 0;
    resp[order[k]] = ok ? R_of[k] : (i64)ORACLE_RESP_NOT_ANALYSED;
  }
  *sched = ok ? 1 : 0;
  if (terms) *terms = g.terms;
  return ORACLE_OK;
}

extern "C" int oracle_gprio_assign_batch(uint32_t n_tasksets, uint32_t n_tasks, uint32_t max_gseg,
                                         const uint32_t *eps_us, const uint32_t *cpu_us,
                                         const uint32_t *period_us, const uint32_t *deadline_us,
                                         const int32_t *prio, const uint8_t *core, const uint8_t *n_gseg,
                                         const uint32_t *gm_us, const uint32_t *ge_us, const uint8_t *skip,
                                         int wait_mode, uint32_t options, int threads, int32_t *gprio,
                                         int64_t *resp, uint8_t *sched, uint64_t *terms_total,
                                         uint32_t *first_bad) {
  if (n_tasksets == 0 || !eps_us || !gprio || !resp || !sched) return ORACLE_EINVAL;
  if (threads < 1) threads = 1;
  if ((uint32_t)threads > n_tasksets) threads = (int)n_tasksets;
  std::vector<int> rc(threads, ORACLE_OK);
  std::vector<uint32_t> bad(threads, 0xffffffffu);
  std::vector<uint64_t> terms(threads, 0);
  auto work = [&](int w) {
    uint32_t lo = (uint32_t)((uint64_t)n_tasksets * w / threads);
    uint32_t hi = (uint32_t)((uint64_t)n_tasksets * (w + 1) / threads);
    for (uint32_t s = lo; s < hi; ++s) {
      size_t to = (size_t)s * n_tasks;
      size_t so = to * max_gseg;
      if (skip && skip[s]) {
        for (uint32_t i = 0; i < n_tasks; ++i) {
          gprio[to + i] = 0;
          resp[to + i] = ORACLE_RESP_NOT_ANALYSED;
        }
        sched[s] = 1;
        continue;
      }
      uint64_t t = 0;
      int r = oracle_gprio_assign_taskset(n_tasks, max_gseg, eps_us[s], cpu_us + to, period_us + to,
                                          deadline_us + to, prio + to, core + to, n_gseg + to,
                                          gm_us ? gm_us + so : nullptr, ge_us ? ge_us + so : nullptr,
                                          wait_mode, options, gprio + to, resp + to, sched + s, &t);
      if (r != ORACLE_OK) {
        rc[w] = r;
        bad[w] = s;
        return;
      }
      terms[w] += t;
    }
  };
  if (threads == 1) {
    work(0);
  } else {
    std::vector<std::thread> pool;
    for (int w = 0; w < threads; ++w) pool.emplace_back(work, w);
    for (auto &th : pool) th.join();
  }
  uint64_t total = 0;
  for (int w = 0; w < threads; ++w) {
    total += terms[w];
    if (rc[w] != ORACLE_OK) {
      if (first_bad) *first_bad = bad[w];
      return rc[w];
    }
  }
  if (terms_total) *terms_total = total;
  return ORACLE_OK;
}

extern "C" int oracle_gprio_rta_batch(uint32_t n_tasksets, uint32_t n_tasks, uint32_t max_gseg,
                                      const uint32_t *eps_us, const uint32_t *cpu_us,
                                      const uint32_t *period_us, const uint32_t *deadline_us,
                                      const int32_t *prio, const uint8_t *core, const uint8_t *n_gseg,
                                      const uint32_t *gm_us, const uint32_t *ge_us, const int32_t *gprio,
                                      int wait_mode, uint32_t options, int64_t *resp, uint8_t *sched,
                                      uint32_t *first_bad) {
  if (n_tasksets == 0 || !eps_us || !gprio || !resp || !sched) return ORACLE_EINVAL;
  for (uint32_t s = 0; s < n_tasksets; ++s) {
    size_t to = (size_t)s * n_tasks;
    size_t so = to * max_gseg;
    int r = oracle_gprio_rta_taskset(n_tasks, max_gseg, eps_us[s], cpu_us + to, period_us + to,
                                     deadline_us + to, prio + to, core + to, n_gseg + to,
                                     gm_us ? gm_us + so : nullptr, ge_us ? ge_us + so : nullptr, gprio + to,
                                     wait_mode, options, resp + to, sched + s, nullptr);
    if (r != ORACLE_OK) {
      if (first_bad) *first_bad = s;
      return r;
    }
  }
  return ORACLE_OK;
}
