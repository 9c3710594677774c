/*
 * Simulation oracle: unit-tick simulator of a multi-core + one-GPU system.
 * TEST INFRASTRUCTURE ONLY.  It is the reference the batched simulator of the GPU
 * library is compared with, and one of the pins of the analysis oracle
 * (rta_oracle.cpp); it shares no code with either.  It executes a concrete
 * schedule one tick at a time and reports the largest response time each task
 * was seen to have (Sec. 6.2 calls it the maximum observed response time); the
 * analytic bounds of Sec. 5 must never be below that.
 *
 * Model (Sec. 2, Sec. 3, Sec. 4.1-4.2, Alg. 1):
 *  - CPU: partitioned, fixed-priority, fully preemptive, one task per core per tick.
 *  - A job is the sequence  c[0], (gm[0], ge[0]), c[1], ..., (gm[eta-1], ge[eta-1]), c[eta]:
 *    CPU segments alternate with GPU segments; a GPU segment is gm ticks of CPU
 *    work (launch, driver calls) followed by ge ticks of pure GPU work.
 *  - While its pure GPU work is outstanding a task either keeps its core
 *    (busy-waiting; it can still be preempted there) or leaves it (self-suspension).
 *  - Round-robin policy: every task with outstanding pure GPU work owns one TSG in
 *    a FIFO ring.  The GPU runs the head TSG for at most L ticks of work, then, if
 *    another TSG waits, spends theta ticks switching and moves the old head to the
 *    tail.  A lone TSG is never switched out.  Work-conserving.
 *  - GCAPS policy: a GPU segment is bracketed by two runlist updates.  An update is
 *    decided by the priority rule of Alg. 1 (real-time tasks only).  An update that
 *    changes the set of running TSGs takes eps ticks on the caller's core, holds the
 *    driver lock and cannot be preempted; its effect on the GPU is applied when it
 *    completes.  An update that leaves the running set unchanged (a lower-priority
 *    task joining the pending list) costs nothing.  The lock is handed to the
 *    highest-priority requester that is able to run on its core.  A task waiting for
 *    the lock sleeps in either waiting mode (Sec. 5.3 names the lock an rt-mutex;
 *    busy-waiting is how a task waits for its GPU work): the lower-priority tasks of
 *    its core run meanwhile.
 *  - Only the task at the head of the running set makes GPU progress.
 *  - Whatever happens at the same instant happens in decreasing CPU priority (equal priorities:
 *    lower caller index first), so a result does not depend on the order the caller lists the tasks in.
 *    Internally the tasks are held in that order; `caller` maps back.
 *
 * Parity: pinned by tests/test_oracle_des.py and tests/test_oracle_sim.py (hand-worked schedules, the
 * motivational example of Sec. 4, closed forms of single-core fixed-priority scheduling, the bounds of
 * Sec. 5 from above, invariance under task permutation).
 */
#include <stdint.h>

#include <algorithm>
#include <deque>
#include <numeric>
#include <thread>
#include <vector>

namespace {

enum Phase { PH_CPU, PH_UPD_BEGIN, PH_GPU, PH_UPD_END };

typedef int64_t tick_t;

struct Op {
  Phase ph;
  tick_t len;
};

struct TaskDef {
  int core, prio, gprio, eta, caller; /* gprio: priority of the GPU segments (Sec. 4.3) */
  tick_t T, offset;
  std::vector<tick_t> c;      /* eta + 1 CPU segments */
  std::vector<tick_t> gm, ge; /* eta GPU segments */
};

struct TaskState {
  std::vector<Op> ops; /* program of one job */
  bool active = false;
  size_t pc = 0;
  tick_t remaining = 0;
  bool in_update = false; /* holds the driver lock, non-preemptible */
  tick_t release = 0;
  tick_t max_resp = 0;
  int64_t jobs_done = 0;
};

struct Sim {
  int n;
  int policy; /* 1 = GCAPS, 2 = round-robin */
  int wait;   /* 0 = busy, 1 = suspend */
  tick_t theta, eps, L;
  std::vector<TaskDef> def;
  std::vector<TaskState> st;
  int n_cores = 0;

  /* GCAPS runlist state (Alg. 1, real-time tasks only) */
  int running = -1;          /* task whose TSGs are on the runlist */
  std::vector<char> pending; /* task_pending */
  int lock_holder = -1;

  /* round-robin ring */
  std::deque<int> ring; /* head = TSG on the GPU */
  tick_t slice_used = 0;
  tick_t switch_left = 0;
  /* Eq. 3 charges a task L + theta per time slice of every *other* TSG (the switch that brings the
   * slice in, and the slice) and nothing for the switch that brings in its own slice.  For tasks
   * flagged here that switch takes no time: the schedule Eq. 3 describes from those tasks' side. */
  std::vector<char> free_switch;
  tick_t switch_into(int i) const { return !free_switch.empty() && free_switch[i] ? 0 : theta; }

  bool overrun = false;

  bool higher(int a, int b) const { return def[a].prio > def[b].prio; }
  /* the runlist decisions of Alg. 1 compare GPU-segment priorities (end of Sec. 4.3) */
  bool higher_g(int a, int b) const { return def[a].gprio > def[b].gprio; }

  void build_program(int i) {
    const TaskDef &d = def[i];
    std::vector<Op> &ops = st[i].ops;
    ops.clear();
    for (int j = 0; j <= d.eta; ++j) {
      ops.push_back({PH_CPU, d.c[j]});
      if (j < d.eta) {
        ops.push_back({PH_CPU, d.gm[j]});
        if (policy == 1) ops.push_back({PH_UPD_BEGIN, 0});
        ops.push_back({PH_GPU, d.ge[j]});
        if (policy == 1) ops.push_back({PH_UPD_END, 0});
      }
    }
  }

  /* Alg. 1, add branch.  Returns true when the running set changes. */
  bool add_changes(int i) const { return running < 0 || higher_g(i, running); }
  void apply_add(int i) {
    if (running < 0) {
      running = i;
    } else if (higher_g(i, running)) {
      pending[running] = 1;
      running = i;
    } else {
      pending[i] = 1;
    }
  }
  /* Alg. 1, remove branch. */
  bool remove_changes(int i) const { return running == i; }
  void apply_remove(int i) {
    if (running == i) {
      int k = -1;
      for (int x = 0; x < n; ++x)
        if (pending[x] && (k < 0 || higher_g(x, k))) k = x;
      running = k;
      if (k >= 0) pending[k] = 0;
    } else {
      pending[i] = 0;
    }
  }

  void enter_phase(int i) {
    TaskState &s = st[i];
    s.remaining = s.ops[s.pc].len;
    if (s.ops[s.pc].ph == PH_GPU && policy == 2 && s.remaining > 0) ring.push_back(i);
  }

  void finish_job(int i, tick_t now_end) {
    TaskState &s = st[i];
    s.active = false;
    s.max_resp = std::max(s.max_resp, now_end - s.release);
    s.jobs_done++;
  }

  /* Advance over everything that takes no time.  `t` is the start of the current tick. */
  void settle(tick_t t) {
    bool moved = true;
    while (moved) {
      moved = false;
      for (int i = 0; i < n; ++i) {
        TaskState &s = st[i];
        if (!s.active || s.in_update) continue;
        Phase ph = s.ops[s.pc].ph;
        bool done = false;
        if ((ph == PH_CPU || ph == PH_GPU) && s.remaining == 0) done = true;
        if (ph == PH_UPD_BEGIN && s.remaining == 0 && lock_holder < 0 && !add_changes(i)) {
          apply_add(i); /* joins the pending list: free */
          done = true;
        }
        if (ph == PH_UPD_END && s.remaining == 0 && lock_holder < 0 && !remove_changes(i)) {
          apply_remove(i);
          done = true;
        }
        if (ph == PH_UPD_BEGIN && s.remaining == 0 && lock_holder < 0 && add_changes(i) && eps == 0) {
          apply_add(i);
          done = true;
        }
        if (ph == PH_UPD_END && s.remaining == 0 && lock_holder < 0 && remove_changes(i) && eps == 0) {
          apply_remove(i);
          done = true;
        }
        if (done) {
          moved = true;
          s.pc++;
          if (s.pc == s.ops.size()) {
            finish_job(i, t);
          } else {
            enter_phase(i);
          }
        }
      }
    }
  }

  bool wants_cpu(int i) const {
    const TaskState &s = st[i];
    if (!s.active) return false;
    Phase ph = s.ops[s.pc].ph;
    if (ph == PH_CPU) return true;
    if (ph == PH_GPU) return wait == 0; /* busy-waiting keeps the core */
    return true;                        /* update phases need the core to issue the call */
  }
  bool is_update_waiter(int i) const {
    const TaskState &s = st[i];
    if (!s.active || s.in_update) return false;
    Phase ph = s.ops[s.pc].ph;
    return ph == PH_UPD_BEGIN || ph == PH_UPD_END;
  }

  void tick(tick_t t) {
    /* releases */
    for (int i = 0; i < n; ++i) {
      if (t >= def[i].offset && (t - def[i].offset) % def[i].T == 0) {
        TaskState &s = st[i];
        if (s.active) {
          overrun = true;
          return;
        }
        s.active = true;
        s.pc = 0;
        s.release = t;
        enter_phase(i);
      }
    }
    settle(t);

    /* CPU arbitration */
    std::vector<int> on_core(n_cores, -1);
    std::vector<char> blocked(n, 0);
    for (int c = 0; c < n_cores; ++c)
      for (int i = 0; i < n; ++i)
        if (def[i].core == c && st[i].active && st[i].in_update) on_core[c] = i;
    auto top_of = [&](int c) {
      int best = -1;
      for (int i = 0; i < n; ++i)
        if (def[i].core == c && wants_cpu(i) && !blocked[i] && (best < 0 || higher(i, best))) best = i;
      return best;
    };
    for (int c = 0; c < n_cores; ++c)
      if (on_core[c] < 0) on_core[c] = top_of(c);
    /* driver lock: highest-priority requester that is at the top of its core */
    if (policy == 1 && lock_holder < 0) {
      int g = -1;
      for (int i = 0; i < n; ++i)
        if (on_core[def[i].core] == i && is_update_waiter(i) && (g < 0 || higher(i, g))) g = i;
      if (g >= 0) {
        lock_holder = g;
        st[g].in_update = true;
        st[g].remaining = eps;
      }
    }
    /* requesters that did not get the lock sleep on it: the core goes to the next task */
    if (policy == 1) {
      for (int c = 0; c < n_cores; ++c) {
        while (on_core[c] >= 0 && is_update_waiter(on_core[c])) {
          blocked[on_core[c]] = 1;
          on_core[c] = top_of(c);
        }
      }
    }

    /* one tick of CPU work */
    for (int c = 0; c < n_cores; ++c) {
      int i = on_core[c];
      if (i < 0) continue;
      TaskState &s = st[i];
      Phase ph = s.ops[s.pc].ph;
      if (s.in_update) {
        s.remaining--;
      } else if (ph == PH_CPU) {
        s.remaining--;
      }
      /* busy GPU wait and lock spin: the core is occupied, nothing advances */
    }

    /* one tick of GPU work */
    if (policy == 1) {
      if (running >= 0) {
        TaskState &s = st[running];
        if (s.active && !s.in_update && s.ops[s.pc].ph == PH_GPU && s.remaining > 0) s.remaining--;
      }
    } else {
      if (switch_left > 0) {
        switch_left--;
      } else if (!ring.empty()) {
        int i = ring.front();
        TaskState &s = st[i];
        s.remaining--;
        slice_used++;
        if (s.remaining == 0) {
          ring.pop_front();
          slice_used = 0;
          if (!ring.empty()) switch_left = switch_into(ring.front());
        } else if (slice_used == L) {
          slice_used = 0;
          if (ring.size() > 1) {
            ring.pop_front();
            ring.push_back(i);
            switch_left = switch_into(ring.front());
          }
        }
      }
    }

    /* completed updates take effect at the end of the tick */
    if (policy == 1 && lock_holder >= 0 && st[lock_holder].remaining == 0) {
      int i = lock_holder;
      TaskState &s = st[i];
      if (s.ops[s.pc].ph == PH_UPD_BEGIN) apply_add(i); else apply_remove(i);
      s.in_update = false;
      lock_holder = -1;
      s.pc++;
      if (s.pc == s.ops.size()) finish_job(i, t + 1); else enter_phase(i);
    }
    /* zero-time follow-ups of what ended in this tick happen at time t + 1 */
    settle(t + 1);
  }
};

/* Runs one schedule over tasks given in caller order; results come back in caller order. */
int run_schedule(std::vector<TaskDef> tasks, int policy, int wait, tick_t theta, tick_t eps, tick_t L,
                 tick_t horizon, tick_t *max_resp, int64_t *jobs_done, const int *free_switch = nullptr) {
  const int n = (int)tasks.size();
  for (int i = 0; i < n; ++i) tasks[i].caller = i;
  std::stable_sort(tasks.begin(), tasks.end(), [](const TaskDef &a, const TaskDef &b) { return a.prio > b.prio; });
  Sim sim;
  sim.n = n;
  sim.policy = policy;
  sim.wait = wait;
  sim.theta = theta;
  sim.eps = eps;
  sim.L = L;
  sim.def = tasks;
  sim.st.resize(n);
  sim.pending.assign(n, 0);
  if (free_switch) {
    sim.free_switch.assign(n, 0);
    for (int i = 0; i < n; ++i) sim.free_switch[i] = free_switch[sim.def[i].caller] != 0;
  }
  for (int i = 0; i < n; ++i) {
    sim.n_cores = std::max(sim.n_cores, sim.def[i].core + 1);
    sim.build_program(i);
  }
  for (tick_t t = 0; t < horizon; ++t) {
    sim.tick(t);
    if (sim.overrun) break;
  }
  for (int i = 0; i < n; ++i) {
    max_resp[sim.def[i].caller] = sim.st[i].max_resp;
    jobs_done[sim.def[i].caller] = sim.st[i].jobs_done;
  }
  return sim.overrun ? 1 : 0;
}

}  // namespace

/*
 * Runs one schedule.  Per-task arrays have n entries; c is [n][max_eta+1], gm/ge
 * are [n][max_eta] (row-major, unused slots ignored).  Releases are strictly
 * periodic from offset[i].  max_resp[i] receives the largest response time of
 * the jobs of task i that completed within `horizon` ticks, jobs_done[i] their
 * number.  Returns 0, or 1 when a job was released while its predecessor was
 * still running (the simulation stops there), or -1 on bad arguments.
 * gprio (may be null: same as prio): priorities of the GPU segments, used by the runlist
 * decisions of the GCAPS policy only.
 * free_switch (may be null: none): round-robin only; the context switch that brings in a time slice of a
 * task with a non-zero entry takes no time, the accounting of Eq. 3 seen from those tasks.
 */
extern "C" int des_run_free(int n, int max_eta, int policy, int wait_mode, int theta, int eps, int L,
                            const int *core, const int *prio, const int *gprio, const int *T, const int *D,
                            const int *offset, const int *eta, const int *c, const int *gm, const int *ge,
                            const int *free_switch, int horizon, int *max_resp, int *jobs_done) {
  (void)D;
  if (n <= 0 || n > 255 || max_eta < 0 || L <= 0 || (policy != 1 && policy != 2) ||
      (wait_mode != 0 && wait_mode != 1))
    return -1;
  std::vector<TaskDef> tasks(n);
  for (int i = 0; i < n; ++i) {
    TaskDef &d = tasks[i];
    d.core = core[i];
    d.prio = prio[i];
    d.gprio = gprio ? gprio[i] : prio[i];
    d.T = T[i];
    d.offset = offset[i];
    d.eta = eta[i];
    if (d.eta > max_eta || d.T <= 0 || d.core < 0 || d.core >= 256) return -1;
    for (int j = 0; j <= d.eta; ++j) d.c.push_back(c[i * (max_eta + 1) + j]);
    for (int j = 0; j < d.eta; ++j) {
      d.gm.push_back(gm[i * max_eta + j]);
      d.ge.push_back(ge[i * max_eta + j]);
    }
  }
  std::vector<tick_t> mr(n);
  std::vector<int64_t> jd(n);
  const int rc = run_schedule(tasks, policy, wait_mode, theta, eps, L, horizon, mr.data(), jd.data(), free_switch);
  for (int i = 0; i < n; ++i) {
    max_resp[i] = (int)mr[i];
    jobs_done[i] = (int)jd[i];
  }
  return rc;
}

extern "C" int des_run_gprio(int n, int max_eta, int policy, int wait_mode, int theta, int eps, int L,
                             const int *core, const int *prio, const int *gprio, const int *T, const int *D,
                             const int *offset, const int *eta, const int *c, const int *gm,
                             const int *ge, int horizon, int *max_resp, int *jobs_done) {
  return des_run_free(n, max_eta, policy, wait_mode, theta, eps, L, core, prio, gprio, T, D, offset, eta, c, gm, ge,
                      nullptr, horizon, max_resp, jobs_done);
}

extern "C" int des_run(int n, int max_eta, int policy, int wait_mode, int theta, int eps, int L,
                       const int *core, const int *prio, const int *T, const int *D,
                       const int *offset, const int *eta, const int *c, const int *gm,
                       const int *ge, int horizon, int *max_resp, int *jobs_done) {
  return des_run_gprio(n, max_eta, policy, wait_mode, theta, eps, L, core, prio, nullptr, T, D, offset, eta, c,
                       gm, ge, horizon, max_resp, jobs_done);
}

/*
 * Simulates every taskset of a batch in the layout of the analysis (per-taskset theta, eps, L; per-task
 * C, T, prio, core, eta^g; per-segment G^m, G^e; one time unit = one tick).  The task model of Sec. 3 gives a
 * job eta^g + 1 CPU segments around its eta^g GPU segments but only their sum C_i; C_i is dealt to them as
 * evenly as integers allow, the first C_i mod (eta^g + 1) segments one tick longer.  offset: [N][n] first
 * release of each task, or null for a synchronous release at time 0.  gprio: [N][n] priorities of the GPU
 * segments (Sec. 4.3: the runlist decisions of GCAPS compare these), or null: the task priorities.  policy_mask: 1 = GCAPS, 2 = round-robin,
 * 3 = both (planes in that order).  Outputs per plane: out_mort [N][n] largest response time of the jobs that
 * completed within `horizon` ticks (0 when none did), out_jobs [N][n] their number, out_flag [N] 1 when a job was
 * released while its predecessor was still running (the simulation of that taskset stops there and the outputs
 * hold what was seen until then), else 0.
 * Returns 0; -1 on bad arguments; -2 when a taskset breaks the task model (T = 0, L = 0, eta^g > S), with
 * *first_bad = its index (else -1).
 */
extern "C" int oracle_simulate_batch(uint32_t N, uint32_t n, uint32_t S, const uint32_t *theta,
                                     const uint32_t *eps, const uint32_t *L, const uint32_t *C, const uint32_t *T,
                                     const int32_t *prio, const uint8_t *core, const uint8_t *n_gseg,
                                     const uint32_t *gm, const uint32_t *ge, const uint32_t *offset,
                                     const int32_t *gprio, int policy_mask, int wait_mode, uint32_t horizon, int threads,
                                     int64_t *out_mort, uint32_t *out_jobs, uint8_t *out_flag, int64_t *first_bad) {
  if (first_bad) *first_bad = -1;
  if (N == 0 || n == 0 || n > 255 || S > 255 || !theta || !eps || !L || !C || !T || !prio || !core || !n_gseg ||
      (S > 0 && (!gm || !ge)) || policy_mask < 1 || policy_mask > 3 || (wait_mode != 0 && wait_mode != 1) ||
      !out_mort || !out_jobs || !out_flag)
    return -1;
  for (uint32_t ts = 0; ts < N; ++ts) {
    bool bad = L[ts] == 0;
    for (uint32_t i = 0; i < n; ++i) bad = bad || T[(size_t)ts * n + i] == 0 || n_gseg[(size_t)ts * n + i] > S;
    if (bad) {
      if (first_bad) *first_bad = ts;
      return -2;
    }
  }
  auto work = [&](uint32_t lo, uint32_t hi) {
    std::vector<tick_t> mr(n);
    std::vector<int64_t> jd(n);
    for (uint32_t ts = lo; ts < hi; ++ts) {
      std::vector<TaskDef> tasks(n);
      for (uint32_t i = 0; i < n; ++i) {
        const size_t at = (size_t)ts * n + i;
        TaskDef &d = tasks[i];
        d.core = core[at];
        d.prio = prio[at];
        d.gprio = gprio ? gprio[at] : prio[at];
        d.T = T[at];
        d.offset = offset ? offset[at] : 0;
        d.eta = n_gseg[at];
        const tick_t parts = d.eta + 1, each = C[at] / parts, longer = C[at] % parts;
        for (int j = 0; j <= d.eta; ++j) d.c.push_back(each + (j < longer ? 1 : 0));
        for (int j = 0; j < d.eta; ++j) {
          d.gm.push_back(gm[at * S + j]);
          d.ge.push_back(ge[at * S + j]);
        }
      }
      int plane = 0;
      for (int policy = 1; policy <= 2; ++policy) {
        if (!(policy_mask & policy)) continue;
        const int rc = run_schedule(tasks, policy, wait_mode, theta[ts], eps[ts], L[ts], horizon, mr.data(), jd.data());
        const size_t base = ((size_t)plane * N + ts) * n;
        for (uint32_t i = 0; i < n; ++i) {
          out_mort[base + i] = mr[i];
          out_jobs[base + i] = (uint32_t)jd[i];
        }
        out_flag[(size_t)plane * N + ts] = (uint8_t)rc;
        ++plane;
      }
    }
  };
  const uint32_t workers = (uint32_t)std::max(1, std::min<int>(threads, (int)N));
  std::vector<std::thread> pool;
  for (uint32_t w = 0; w < workers; ++w)
    pool.emplace_back(work, (uint32_t)((uint64_t)N * w / workers), (uint32_t)((uint64_t)N * (w + 1) / workers));
  for (auto &th : pool) th.join();
  return 0;
}
