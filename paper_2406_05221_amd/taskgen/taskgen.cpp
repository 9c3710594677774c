/*
 * Seeded synthetic taskset generator (host only).  It produces INPUTS in the
 * task model of Sec. 3 following the generation recipe of Sec. 6.1 (number of
 * tasks per CPU, UUniFast utilisation split per CPU, uniformly drawn period and
 * number of GPU segments, rate-monotonic priorities); it contains none of the
 * response-time analysis.  Both the CPU oracle's tests and the GPU library's
 * tests and benchmark draw their inputs from here.
 *
 * Every taskset is generated from its own counter-based stream
 * (seed, stream id, taskset index) -> splitmix64, so any taskset can be
 * regenerated alone and the result does not depend on the thread count.
 *
 * The library's device generator (csrc/taskgen_device.hip.inc) produces the same batches bit for
 * bit.  What makes that possible: the random stream is integer arithmetic; every real-valued step
 * is a fixed sequence of IEEE-754 double additions, multiplications and divisions (correctly
 * rounded on both machines; no fused multiply-add: this file is built with -ffp-contract=off);
 * and logarithm and power are the two routines below, not a math library's.
 */
#include <stdint.h>

#include <algorithm>
#include <cmath>
#include <thread>
#include <vector>

namespace {

struct Rng {
  uint64_t s;
  static uint64_t mix(uint64_t z) {
    z = (z ^ (z >> 30)) * 0xBF58476D1CE4E5B9ull;
    z = (z ^ (z >> 27)) * 0x94D049BB133111EBull;
    return z ^ (z >> 31);
  }
  Rng(uint64_t seed, uint64_t stream, uint64_t index) {
    s = mix(seed + 0x9E3779B97F4A7C15ull);
    s = mix(s ^ (stream + 0x632BE59BD9B4E019ull));
    s = mix(s ^ (index * 0xD1342543DE82EF95ull + 1));
  }
  uint64_t next() { /* splitmix64 */
    s += 0x9E3779B97F4A7C15ull;
    return mix(s);
  }
  double uniform() { return (double)(next() >> 11) * (1.0 / 9007199254740992.0); } /* [0,1) */
  double uniform(double lo, double hi) { return lo + (hi - lo) * uniform(); }
  uint32_t integer(uint32_t lo, uint32_t hi) { /* inclusive */
    return lo + (uint32_t)(uniform() * (double)(hi - lo + 1));
  }
};

/*
 * log2(x) for a finite x > 0 and 2^x for |x| < 1000, to about 1e-13: enough for drawing periods
 * and utilisations, and the same bits wherever IEEE double arithmetic is.
 *   x = m 2^e, m in (sqrt(1/2), sqrt(2)]:  log2 x = e + (2/ln 2) t (1 + t^2/3 + ... + t^14/15), t = (m-1)/(m+1)
 *   x = i + f, f in [0,1):                 2^x = 2^i sum_{k <= 14} z^k / k!, z = f ln 2 (Horner's rule)
 */
double gen_log2(double x) {
  uint64_t bits;
  static_assert(sizeof bits == sizeof x, "IEEE double");
  __builtin_memcpy(&bits, &x, sizeof bits);
  int e = (int)((bits >> 52) & 0x7ff) - 1023;
  bits = (bits & 0x000fffffffffffffull) | 0x3ff0000000000000ull;
  double m;
  __builtin_memcpy(&m, &bits, sizeof m);
  if (m > 1.4142135623730951) {
    m = m * 0.5;
    e += 1;
  }
  const double t = (m - 1.0) / (m + 1.0), t2 = t * t;
  double p = 1.0 / 15.0;
  p = p * t2 + 1.0 / 13.0;
  p = p * t2 + 1.0 / 11.0;
  p = p * t2 + 1.0 / 9.0;
  p = p * t2 + 1.0 / 7.0;
  p = p * t2 + 1.0 / 5.0;
  p = p * t2 + 1.0 / 3.0;
  p = p * t2 + 1.0;
  return (double)e + 2.8853900817779268 * (t * p);
}

double gen_exp2(double x) {
  const double fl = std::floor(x);
  const double z = (x - fl) * 0.6931471805599453;
  /* sum_{k <= 14} z^k / k! by Horner's rule; the constants are 1/k! rounded to double */
  double p = 1.1470745597729725e-11;
  p = p * z + 1.6059043836821613e-10;
  p = p * z + 2.08767569878681e-09;
  p = p * z + 2.505210838544172e-08;
  p = p * z + 2.755731922398589e-07;
  p = p * z + 2.7557319223985893e-06;
  p = p * z + 2.48015873015873e-05;
  p = p * z + 0.0001984126984126984;
  p = p * z + 0.001388888888888889;
  p = p * z + 0.008333333333333333;
  p = p * z + 0.041666666666666664;
  p = p * z + 0.16666666666666666;
  p = p * z + 0.5;
  p = p * z + 1.0;
  p = p * z + 1.0;
  uint64_t bits;
  __builtin_memcpy(&bits, &p, sizeof bits); /* p in [1, 2]: scaling by 2^i is an add to the exponent */
  bits += (uint64_t)((int64_t)fl) << 52;
  __builtin_memcpy(&p, &bits, sizeof p);
  return p;
}

/* r^(1/k) for r in [0, 1) */
double gen_root(double r, uint32_t k) { return r > 0.0 ? gen_exp2(gen_log2(r) / (double)k) : 0.0; }

struct Spec {
  uint64_t seed, stream, first_index;
  uint32_t n_tasksets, n_cores, tasks_per_core, max_gseg;
  double util_lo, util_hi;
  const double *util_fixed; /* per taskset, or null */
  uint32_t eta_lo, eta_hi;
  double share_lo, share_hi;
  const double *share_fixed;
  uint32_t t_lo, t_hi;
  uint32_t ovh_lo, ovh_hi;
  const uint32_t *ovh_fixed;
  uint32_t slice;
  const uint32_t *slice_fixed;
};

struct Out {
  uint32_t *theta, *eps, *slice, *cpu, *period, *deadline;
  int32_t *prio;
  uint8_t *core, *n_gseg;
  uint32_t *gm, *ge;
};

void one_taskset(const Spec &sp, const Out &o, uint32_t k) {
  Rng rng(sp.seed, sp.stream, sp.first_index + k);
  const uint32_t n = sp.n_cores * sp.tasks_per_core;
  const uint32_t S = sp.max_gseg;
  const size_t to = (size_t)k * n;

  uint32_t ovh = sp.ovh_fixed ? sp.ovh_fixed[k] : rng.integer(sp.ovh_lo, sp.ovh_hi);
  o.theta[k] = ovh;
  o.eps[k] = ovh;
  o.slice[k] = sp.slice_fixed ? sp.slice_fixed[k] : sp.slice;

  const double l2_lo = gen_log2((double)sp.t_lo), l2_hi = gen_log2((double)sp.t_hi);
  for (uint32_t c = 0; c < sp.n_cores; ++c) {
    double U = sp.util_fixed ? sp.util_fixed[k] : rng.uniform(sp.util_lo, sp.util_hi);
    /* UUniFast: utilisations of the tasks of this core, summing to U */
    double sum = U;
    for (uint32_t j = 0; j < sp.tasks_per_core; ++j) {
      const uint32_t i = c * sp.tasks_per_core + j;
      double u;
      if (j + 1 < sp.tasks_per_core) {
        double next = sum * gen_root(rng.uniform(), sp.tasks_per_core - 1 - j);
        u = sum - next;
        sum = next;
      } else {
        u = sum;
      }
      double t = std::floor(gen_exp2(rng.uniform(l2_lo, l2_hi))); /* log-uniform */
      uint32_t T = (uint32_t)std::min((double)sp.t_hi, std::max((double)sp.t_lo, t));
      uint32_t eta = rng.integer(sp.eta_lo, sp.eta_hi);
      uint32_t W = (uint32_t)std::floor(u * (double)T + 0.5); /* total WCET C + G */
      W = std::max(W, 2 * eta + 1);
      double share = sp.share_fixed ? sp.share_fixed[k] : rng.uniform(sp.share_lo, sp.share_hi);
      uint32_t g = (uint32_t)std::floor(share * (double)W + 0.5);
      g = std::min(std::max(g, 2 * eta), W - 1);
      if (eta == 0) g = 0; /* a CPU-only task keeps its whole demand as CPU time */
      o.cpu[to + i] = W - g;
      o.period[to + i] = T;
      o.deadline[to + i] = T;
      o.core[to + i] = (uint8_t)c;
      o.n_gseg[to + i] = (uint8_t)eta;
      for (uint32_t s = 0; s < S; ++s) {
        uint32_t gj = 0;
        if (s < eta) gj = g / eta + (s < g % eta ? 1 : 0);
        o.gm[(to + i) * S + s] = gj / 2;      /* launch / copy half */
        o.ge[(to + i) * S + s] = gj - gj / 2; /* kernel half */
      }
    }
  }
  /* rate-monotonic priorities over the whole taskset: shorter period = higher,
   * equal periods: lower index higher.  Larger value = higher priority. */
  for (uint32_t i = 0; i < n; ++i) {
    uint32_t rank = 0;
    for (uint32_t j = 0; j < n; ++j)
      if (o.period[to + j] < o.period[to + i] || (o.period[to + j] == o.period[to + i] && j < i)) ++rank;
    o.prio[to + i] = (int32_t)(n - rank);
  }
}

}  // namespace

extern "C" int taskgen_generate(uint64_t seed, uint64_t stream, uint64_t first_index,
                                uint32_t n_tasksets, uint32_t n_cores, uint32_t tasks_per_core,
                                uint32_t max_gseg, double util_lo, double util_hi,
                                const double *util_fixed, uint32_t eta_lo, uint32_t eta_hi,
                                double share_lo, double share_hi, const double *share_fixed,
                                uint32_t t_lo, uint32_t t_hi, uint32_t ovh_lo, uint32_t ovh_hi,
                                const uint32_t *ovh_fixed, uint32_t slice, const uint32_t *slice_fixed,
                                int threads, uint32_t *theta_us, uint32_t *eps_us, uint32_t *slice_us,
                                uint32_t *cpu_us, uint32_t *period_us, uint32_t *deadline_us,
                                int32_t *prio, uint8_t *core, uint8_t *n_gseg, uint32_t *gm_us,
                                uint32_t *ge_us) {
  if (n_tasksets == 0 || n_cores == 0 || n_cores > 255 || tasks_per_core == 0 ||
      n_cores * tasks_per_core > 255 || eta_lo > eta_hi || eta_hi > max_gseg || t_lo == 0 ||
      t_lo > t_hi || ovh_lo > ovh_hi || util_lo > util_hi || share_lo > share_hi)
    return -1;
  Spec sp{seed, stream, first_index, n_tasksets, n_cores, tasks_per_core, max_gseg, util_lo, util_hi,
          util_fixed, eta_lo, eta_hi, share_lo, share_hi, share_fixed, t_lo, t_hi, ovh_lo, ovh_hi,
          ovh_fixed, slice, slice_fixed};
  Out o{theta_us, eps_us, slice_us, cpu_us, period_us, deadline_us, prio, core, n_gseg, gm_us, ge_us};
  if (threads < 1) threads = 1;
  if ((uint32_t)threads > n_tasksets) threads = (int)n_tasksets;
  auto work = [&](int w) {
    uint32_t lo = (uint32_t)((uint64_t)n_tasksets * w / threads);
    uint32_t hi = (uint32_t)((uint64_t)n_tasksets * (w + 1) / threads);
    for (uint32_t k = lo; k < hi; ++k) one_taskset(sp, o, k);
  };
  if (threads == 1) {
    work(0);
  } else {
    std::vector<std::thread> pool;
    for (int w = 0; w < threads; ++w) pool.emplace_back(work, w);
    for (auto &t : pool) t.join();
  }
  return 0;
}

namespace {

/* Parameters of the schedulability experiments (Sec. 6.1, Table 3); ranges are inclusive. */
struct Table3 {
  uint64_t seed, stream, first_index;
  uint32_t n_tasksets, n_cpus, per_cpu_lo, per_cpu_hi, max_gseg;
  double gpu_ratio_lo, gpu_ratio_hi; /* share of GPU-using tasks in a taskset */
  double util_lo, util_hi;           /* utilisation per CPU */
  uint32_t t_lo, t_hi;               /* period, microseconds, drawn uniformly */
  uint32_t eta_lo, eta_hi;           /* GPU segments of a GPU-using task */
  double gc_lo, gc_hi;               /* G_i / C_i */
  double gm_lo, gm_hi;               /* G^m_i / G_i */
  uint32_t theta, eps, slice;
};

/* One taskset into row k of arrays laid out for n_max = n_cpus * per_cpu_hi tasks; the first
 * count[k] slots of the row are the tasks (the rest is zero). */
void one_table3(const Table3 &sp, const Out &o, uint32_t *count, uint32_t k) {
  Rng rng(sp.seed, sp.stream, sp.first_index + k);
  const uint32_t n_max = sp.n_cpus * sp.per_cpu_hi, S = sp.max_gseg;
  const size_t to = (size_t)k * n_max;
  o.theta[k] = sp.theta;
  o.eps[k] = sp.eps;
  o.slice[k] = sp.slice;
  for (uint32_t i = 0; i < n_max; ++i) {
    o.cpu[to + i] = o.period[to + i] = o.deadline[to + i] = 0;
    o.prio[to + i] = 0;
    o.core[to + i] = o.n_gseg[to + i] = 0;
    for (uint32_t s = 0; s < S; ++s) o.gm[(to + i) * S + s] = o.ge[(to + i) * S + s] = 0;
  }
  /* number of tasks on each CPU, then the utilisation of each task: UUniFast per CPU */
  std::vector<double> util;
  for (uint32_t c = 0; c < sp.n_cpus; ++c) {
    const uint32_t m = rng.integer(sp.per_cpu_lo, sp.per_cpu_hi);
    double sum = rng.uniform(sp.util_lo, sp.util_hi);
    for (uint32_t j = 0; j < m; ++j) {
      double u = sum;
      if (j + 1 < m) {
        const double next = sum * gen_root(rng.uniform(), m - 1 - j);
        u = sum - next;
        sum = next;
      }
      util.push_back(u);
    }
  }
  const uint32_t n = (uint32_t)util.size();
  count[k] = n;
  /* which tasks use the GPU: round(ratio * n) of them, chosen by a partial shuffle */
  const double ratio = rng.uniform(sp.gpu_ratio_lo, sp.gpu_ratio_hi);
  const uint32_t n_gpu = std::min(n, (uint32_t)std::floor(ratio * (double)n + 0.5));
  std::vector<uint32_t> pick(n);
  for (uint32_t i = 0; i < n; ++i) pick[i] = i;
  std::vector<char> uses_gpu(n, 0);
  for (uint32_t i = 0; i < n_gpu; ++i) {
    std::swap(pick[i], pick[rng.integer(i, n - 1)]);
    uses_gpu[pick[i]] = 1;
  }
  for (uint32_t i = 0; i < n; ++i) {
    const uint32_t T = rng.integer(sp.t_lo, sp.t_hi);
    const uint32_t eta = uses_gpu[i] ? rng.integer(sp.eta_lo, sp.eta_hi) : 0u;
    uint32_t W = (uint32_t)std::floor(util[i] * (double)T + 0.5); /* C_i + G_i */
    W = std::max(W, 2 * eta + 1);
    uint32_t g = 0;
    if (eta > 0) {
      const double gc = rng.uniform(sp.gc_lo, sp.gc_hi);
      g = (uint32_t)std::floor((double)W * gc / (1.0 + gc) + 0.5);
      g = std::min(std::max(g, 2 * eta), W - 1);
    }
    const double gm_share = eta > 0 ? rng.uniform(sp.gm_lo, sp.gm_hi) : 0.0;
    o.cpu[to + i] = W - g;
    o.period[to + i] = T;
    o.deadline[to + i] = T;
    o.n_gseg[to + i] = (uint8_t)eta;
    for (uint32_t s = 0; s < eta; ++s) {
      const uint32_t gj = g / eta + (s < g % eta ? 1 : 0); /* >= 2 */
      uint32_t m = (uint32_t)std::floor(gm_share * (double)gj + 0.5);
      m = std::min(m, gj - 1);
      o.gm[(to + i) * S + s] = m;
      o.ge[(to + i) * S + s] = gj - m;
    }
  }
  /* rate-monotonic priorities: shorter period = higher; equal periods: lower index higher */
  for (uint32_t i = 0; i < n; ++i) {
    uint32_t rank = 0;
    for (uint32_t j = 0; j < n; ++j)
      if (o.period[to + j] < o.period[to + i] || (o.period[to + j] == o.period[to + i] && j < i)) ++rank;
    o.prio[to + i] = (int32_t)(n - rank);
  }
  /* re-allocation to the CPUs, worst-fit decreasing: tasks by decreasing utilisation (ties: lower
   * index first), each to the CPU with the smallest load so far (ties: lower CPU first) */
  std::vector<uint32_t> by_util(n);
  for (uint32_t i = 0; i < n; ++i) by_util[i] = i;
  std::stable_sort(by_util.begin(), by_util.end(), [&](uint32_t a, uint32_t b) { return util[a] > util[b]; });
  std::vector<double> load(sp.n_cpus, 0.0);
  for (uint32_t i : by_util) {
    uint32_t best = 0;
    for (uint32_t c = 1; c < sp.n_cpus; ++c)
      if (load[c] < load[best]) best = c;
    o.core[to + i] = (uint8_t)best;
    load[best] += util[i];
  }
}

}  // namespace

/*
 * Tasksets by the recipe of the schedulability experiments (Sec. 6.1, Table 3).  Arrays are laid
 * out for n_max = n_cpus * per_cpu_hi tasks per taskset; n_tasks[k] says how many of row k are
 * tasks.  Returns 0, or -1 on invalid parameters.
 */
extern "C" int taskgen_table3(uint64_t seed, uint64_t stream, uint64_t first_index, uint32_t n_tasksets,
                              uint32_t n_cpus, uint32_t per_cpu_lo, uint32_t per_cpu_hi, uint32_t max_gseg,
                              double gpu_ratio_lo, double gpu_ratio_hi, double util_lo, double util_hi,
                              uint32_t t_lo, uint32_t t_hi, uint32_t eta_lo, uint32_t eta_hi, double gc_lo,
                              double gc_hi, double gm_lo, double gm_hi, uint32_t theta, uint32_t eps,
                              uint32_t slice, int threads, uint32_t *n_tasks, uint32_t *theta_us,
                              uint32_t *eps_us, uint32_t *slice_us, uint32_t *cpu_us, uint32_t *period_us,
                              uint32_t *deadline_us, int32_t *prio, uint8_t *core, uint8_t *n_gseg,
                              uint32_t *gm_us, uint32_t *ge_us) {
  if (n_tasksets == 0 || n_cpus == 0 || n_cpus > 255 || per_cpu_lo == 0 || per_cpu_lo > per_cpu_hi ||
      n_cpus * per_cpu_hi > 255 || eta_lo == 0 || eta_lo > eta_hi || eta_hi > max_gseg || t_lo == 0 || t_lo > t_hi ||
      util_lo > util_hi || util_lo <= 0.0 || gpu_ratio_lo > gpu_ratio_hi || gpu_ratio_lo < 0.0 || gpu_ratio_hi > 1.0 ||
      gc_lo > gc_hi || gc_lo < 0.0 || gm_lo > gm_hi || gm_lo < 0.0 || gm_hi > 1.0 || slice == 0)
    return -1;
  Table3 sp{seed, stream, first_index, n_tasksets, n_cpus, per_cpu_lo, per_cpu_hi, max_gseg, gpu_ratio_lo,
            gpu_ratio_hi, util_lo, util_hi, t_lo, t_hi, eta_lo, eta_hi, gc_lo, gc_hi, gm_lo, gm_hi, theta, eps, slice};
  Out o{theta_us, eps_us, slice_us, cpu_us, period_us, deadline_us, prio, core, n_gseg, gm_us, ge_us};
  if (threads < 1) threads = 1;
  if ((uint32_t)threads > n_tasksets) threads = (int)n_tasksets;
  auto work = [&](int w) {
    uint32_t lo = (uint32_t)((uint64_t)n_tasksets * w / threads);
    uint32_t hi = (uint32_t)((uint64_t)n_tasksets * (w + 1) / threads);
    for (uint32_t k = lo; k < hi; ++k) one_table3(sp, o, n_tasks, k);
  };
  if (threads == 1) {
    work(0);
  } else {
    std::vector<std::thread> pool;
    for (int w = 0; w < threads; ++w) pool.emplace_back(work, w);
    for (auto &t : pool) t.join();
  }
  return 0;
}
