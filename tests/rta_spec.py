"""A second, independent write-up of the response-time recurrences, component by component
(P^C, B^C, I^dp, I^id, I^ie of Eq. 1, 2, 4) in set notation with unbounded Python integers.
Used only by the tests: to search the least fixed point exhaustively and to cross-check the
C++ oracle's iteration.  It is not a pin by itself (it restates the same lemmas)."""


def cdiv(a, b):
    return -(-a // b)


class Spec:
    def __init__(self, tasks, theta, eps, L):
        """tasks: priority order (index 0 highest); dicts with C, T, D, core, gm[], ge[]."""
        self.t = tasks
        self.theta, self.eps, self.L = theta, eps, L
        self.R = {}

    # task-level quantities (Sec. 3)
    def eta(self, i): return len(self.t[i]["ge"])
    def gpu(self, i): return self.eta(i) > 0
    def C(self, i): return self.t[i]["C"]
    def T(self, i): return self.t[i]["T"]
    def Gm(self, i): return sum(self.t[i]["gm"])
    def Ge(self, i): return sum(self.t[i]["ge"])
    def G(self, i): return self.Gm(i) + self.Ge(i)
    def hp(self, i): return set(range(i))
    def hpp(self, i): return {h for h in range(i) if self.t[h]["core"] == self.t[i]["core"]}
    def gpu_tasks(self): return {k for k in range(len(self.t)) if self.gpu(k)}
    # Sec. 5.3 starred demands, jitters
    def Ge_star(self, h): return self.Ge(h) + 2 * self.eps * self.eta(h)
    def Gm_star(self, h): return self.Gm(h) + 2 * self.eps * self.eta(h)
    def Jc(self, h): return self.R[h] - (self.C(h) + self.Gm(h))
    def Jg(self, h): return self.R[h] - self.Ge(h)

    def interleave(self, nu, ge):  # Eq. 3
        return (self.L + self.theta) * nu * cdiv(ge, self.L)

    def components(self, i, R, policy, wait):
        """Returns dict of the interference components for window R."""
        hpp, hp = self.hpp(i), self.hp(i)
        remote = hp - hpp
        gi = self.gpu(i)
        PC = BC = Idp = Iid = Iie = 0
        if policy == 2:  # round-robin driver
            Iie = sum(self.interleave(len(self.gpu_tasks() - {i}), ge) for ge in self.t[i]["ge"])
            if wait == 0:
                PC = sum(cdiv(R, self.T(h)) * (self.C(h) + self.Gm(h)) for h in hpp)
                nu = len((self.gpu_tasks() - hpp)) + 1
                Iid = sum(cdiv(R, self.T(h)) * sum(self.interleave(nu, ge) for ge in self.t[h]["ge"])
                          for h in hpp if self.gpu(h))
            else:
                PC = sum(cdiv(R + (self.Jc(h) if self.gpu(h) else 0), self.T(h)) * (self.C(h) + self.Gm(h))
                         for h in hpp)
        else:  # GCAPS
            BC = (self.eta(i) + 1) * self.eps
            if wait == 0:
                PC = sum(cdiv(R, self.T(h)) * (self.C(h) + self.Gm(h)) for h in hpp)
                same = sum(cdiv(R, self.T(h)) * self.Ge_star(h) for h in hpp if self.gpu(h))
                far = sum(cdiv(R + self.Jg(h), self.T(h)) * self.Ge_star(h) for h in remote if self.gpu(h))
                if gi:
                    Idp = same + far
                else:
                    Idp = same  # reading: the busy-wait of a same-core task delays CPU-only tasks too
                    Iid = far
            else:
                PC = (sum(cdiv(R, self.T(h)) * self.C(h) for h in hpp if not self.gpu(h)) +
                      sum(cdiv(R + self.Jc(h), self.T(h)) * (self.C(h) + self.Gm_star(h)) for h in hpp if self.gpu(h)))
                if gi:
                    Idp = (sum(cdiv(R + self.Jg(h), self.T(h)) * self.Ge(h) for h in hpp if self.gpu(h)) +
                           sum(cdiv(R + self.Jg(h), self.T(h)) * self.Ge_star(h) for h in remote if self.gpu(h)))
        return dict(PC=PC, BC=BC, Idp=Idp, Iid=Iid, Iie=Iie)

    def own(self, i, policy):
        return self.C(i) + self.G(i) + (2 * self.eps * self.eta(i) if policy == 1 else 0)

    def rhs(self, i, R, policy, wait):
        return self.own(i, policy) + sum(self.components(i, R, policy, wait).values())

    def least_fixed_points(self, policy, wait):
        """Exhaustive search: smallest r in [0, D_i] with rhs(r) == r (equivalently rhs(r) <= r)."""
        out = []
        self.R = {}
        for i in range(len(self.t)):
            found = None
            for r in range(0, self.t[i]["D"] + 1):
                if self.rhs(i, r, policy, wait) <= r:
                    found = r
                    break
            if found is None:
                out.append(-1)
                out.extend([-2] * (len(self.t) - i - 1))
                return out
            self.R[i] = found
            out.append(found)
        return out
