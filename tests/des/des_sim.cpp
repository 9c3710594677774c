/*
 * Discrete-event (unit-tick) simulator of a tiny multi-core + one-GPU system.
 * TEST TOOL ONLY: it is one of the pins of the CPU oracle and shares no code
 * with the oracle or with the GPU library.  It executes a concrete schedule and
 * reports the largest response time each task was seen to have; the analytic
 * bounds of Sec. 5 must never be below that.
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
 *    the lock behaves like a task waiting for the GPU (spins or sleeps).
 *  - Only the task at the head of the running set makes GPU progress.
 */
#include <stdint.h>

#include <algorithm>
#include <deque>
#include <vector>

namespace {

enum Phase { PH_CPU, PH_UPD_BEGIN, PH_GPU, PH_UPD_END };

struct Op {
  Phase ph;
  int len;
};

struct TaskDef {
  int core, prio, gprio, T, D, offset, eta; /* gprio: priority of the GPU segments (Sec. 4.3) */
  std::vector<int> c;      /* eta + 1 CPU segments */
  std::vector<int> gm, ge; /* eta GPU segments */
};

struct TaskState {
  std::vector<Op> ops; /* program of one job */
  bool active = false;
  size_t pc = 0;
  int remaining = 0;
  bool in_update = false; /* holds the driver lock, non-preemptible */
  int release = 0;
  int max_resp = 0;
  int jobs_done = 0;
};

struct Sim {
  int n;
  int policy; /* 1 = GCAPS, 2 = round-robin */
  int wait;   /* 0 = busy, 1 = suspend */
  int theta, eps, L;
  std::vector<TaskDef> def;
  std::vector<TaskState> st;
  int n_cores = 0;

  /* GCAPS runlist state (Alg. 1, real-time tasks only) */
  int running = -1;          /* task whose TSGs are on the runlist */
  std::vector<char> pending; /* task_pending */
  int lock_holder = -1;

  /* round-robin ring */
  std::deque<int> ring; /* head = TSG on the GPU */
  int slice_used = 0;
  int switch_left = 0;

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

  void finish_job(int i, int now_end) {
    TaskState &s = st[i];
    s.active = false;
    s.max_resp = std::max(s.max_resp, now_end - s.release);
    s.jobs_done++;
  }

  /* Advance over everything that takes no time.  `t` is the start of the current tick. */
  void settle(int t) {
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

  void tick(int t) {
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
      for (int c = 0; c < n_cores; ++c) {
        int i = on_core[c];
        if (i >= 0 && is_update_waiter(i) && (g < 0 || higher(i, g))) g = i;
      }
      if (g >= 0) {
        lock_holder = g;
        st[g].in_update = true;
        st[g].remaining = eps;
      }
    }
    /* requesters that did not get the lock: spin (busy) or step aside (suspend) */
    if (policy == 1 && wait == 1) {
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
          if (!ring.empty()) switch_left = theta;
        } else if (slice_used == L) {
          slice_used = 0;
          if (ring.size() > 1) {
            ring.pop_front();
            ring.push_back(i);
            switch_left = theta;
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
 */
extern "C" int des_run_gprio(int n, int max_eta, int policy, int wait_mode, int theta, int eps, int L,
                             const int *core, const int *prio, const int *gprio, const int *T, const int *D,
                             const int *offset, const int *eta, const int *c, const int *gm,
                             const int *ge, int horizon, int *max_resp, int *jobs_done) {
  if (n <= 0 || n > 16 || max_eta < 0 || L <= 0 || (policy != 1 && policy != 2) ||
      (wait_mode != 0 && wait_mode != 1))
    return -1;
  Sim sim;
  sim.n = n;
  sim.policy = policy;
  sim.wait = wait_mode;
  sim.theta = theta;
  sim.eps = eps;
  sim.L = L;
  sim.def.resize(n);
  sim.st.resize(n);
  sim.pending.assign(n, 0);
  for (int i = 0; i < n; ++i) {
    TaskDef &d = sim.def[i];
    d.core = core[i];
    d.prio = prio[i];
    d.gprio = gprio ? gprio[i] : prio[i];
    d.T = T[i];
    d.D = D[i];
    d.offset = offset[i];
    d.eta = eta[i];
    if (d.eta > max_eta || d.T <= 0 || d.core < 0 || d.core >= 64) return -1;
    sim.n_cores = std::max(sim.n_cores, d.core + 1);
    for (int j = 0; j <= d.eta; ++j) d.c.push_back(c[i * (max_eta + 1) + j]);
    for (int j = 0; j < d.eta; ++j) {
      d.gm.push_back(gm[i * max_eta + j]);
      d.ge.push_back(ge[i * max_eta + j]);
    }
    sim.build_program(i);
  }
  for (int t = 0; t < horizon; ++t) {
    sim.tick(t);
    if (sim.overrun) break;
  }
  for (int i = 0; i < n; ++i) {
    max_resp[i] = sim.st[i].max_resp;
    jobs_done[i] = sim.st[i].jobs_done;
  }
  return sim.overrun ? 1 : 0;
}

extern "C" int des_run(int n, int max_eta, int policy, int wait_mode, int theta, int eps, int L,
                       const int *core, const int *prio, const int *T, const int *D,
                       const int *offset, const int *eta, const int *c, const int *gm,
                       const int *ge, int horizon, int *max_resp, int *jobs_done) {
  return des_run_gprio(n, max_eta, policy, wait_mode, theta, eps, L, core, prio, nullptr, T, D, offset, eta, c,
                       gm, ge, horizon, max_resp, jobs_done);
}
