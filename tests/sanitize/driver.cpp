/*
 * Host-only driver for sanitizer builds (AddressSanitizer + UndefinedBehaviorSanitizer): the host generator,
 * the analysis oracle and the simulation oracle, compiled from their sources into one program and run over
 * generated batches, including values near the top of the 32-bit range where the saturating 64-bit arithmetic of
 * the analysis is at work.  Prints "ok" when every call returned what it should.  TEST INFRASTRUCTURE ONLY.
 */
#include "../../paper_2406_05221_amd/taskgen/taskgen.cpp"
#include "../../oracle/rta_oracle.cpp"
#include "../../oracle/sim_oracle.cpp"

#include <cstdio>

int main() {
  const uint32_t N = 600, cores = 3, per = 4, n = cores * per, S = 3;
  std::vector<uint32_t> theta(N), eps(N), L(N), C(N * n), T(N * n), D(N * n), gm(N * n * S), ge(N * n * S);
  std::vector<int32_t> prio(N * n), gprio(N * n);
  std::vector<uint8_t> core(N * n), eta(N * n), sched(2 * N), skip(N, 0), flag(2 * N);
  std::vector<int64_t> resp(2 * (size_t)N * n), mort(2 * (size_t)N * n);
  std::vector<uint32_t> jobs(2 * (size_t)N * n);
  int bad = 0;
  for (int pass = 0; pass < 3; ++pass) {
    /* pass 0: microsecond-scale values; pass 1: small values (the simulator walks them tick by tick);
     * pass 2: periods and demands near 2^32 */
    const uint32_t t_lo = pass == 0 ? 1000u : (pass == 1 ? 30u : 3000000000u);
    const uint32_t t_hi = pass == 0 ? 1000000u : (pass == 1 ? 300u : 4294967295u);
    if (taskgen_generate(7, 40 + pass, 0, N, cores, per, S, 0.2, 0.9, nullptr, 0, S, 0.1, 0.6, nullptr, t_lo, t_hi,
                         pass == 1 ? 0 : 50, pass == 1 ? 3 : 500, nullptr, pass == 1 ? 8 : 1024, nullptr, 4,
                         theta.data(), eps.data(), L.data(), C.data(), T.data(), D.data(), prio.data(), core.data(),
                         eta.data(), gm.data(), ge.data()) != 0)
      bad |= 1;
    for (int wait = 0; wait < 2; ++wait)
      for (uint32_t options = 0; options < 4; ++options) {
        uint64_t terms = 0;
        uint32_t first = 0;
        if (oracle_rta_batch(N, n, S, theta.data(), eps.data(), L.data(), C.data(), T.data(), D.data(), prio.data(),
                             core.data(), eta.data(), gm.data(), ge.data(), 3, wait, options, 4, resp.data(),
                             sched.data(), &terms, &first) != 0)
          bad |= 2;
      }
    for (int wait = 0; wait < 2; ++wait) {
      uint64_t terms = 0;
      uint32_t first = 0;
      if (oracle_gprio_assign_batch(N, n, S, eps.data(), C.data(), T.data(), D.data(), prio.data(), core.data(),
                                    eta.data(), gm.data(), ge.data(), skip.data(), wait, 0, 4, gprio.data(), resp.data(),
                                    sched.data(), &terms, &first) != 0)
        bad |= 4;
    }
    if (pass == 1)
      for (int wait = 0; wait < 2; ++wait) {
        int64_t first = 0;
        if (oracle_simulate_batch(N, n, S, theta.data(), eps.data(), L.data(), C.data(), T.data(), prio.data(),
                                  core.data(), eta.data(), gm.data(), ge.data(), nullptr, wait ? gprio.data() : nullptr, 3,
                                  wait, 1500, 4, mort.data(), jobs.data(), flag.data(), &first) != 0)
          bad |= 8;
      }
  }
  std::printf(bad ? "failed %d\n" : "ok\n", bad);
  return bad;
}
