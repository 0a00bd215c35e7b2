"""CPU oracle of the parallelism planner (Sec. 3.3).  TEST INFRASTRUCTURE ONLY.

Plain Python, one function per formula or algorithm step, in the paper's notation:

  stage_memory          Eq. (3)   Mem_p(beta) = MOD + OPT + K_p * ACT(beta)
  allreduce_time        Eq. (5)   T_a^s
  round_latency         Eq. (4), Eq. (5) (T_w^s), Eq. (6) (T_e^s around the dominant step)
  capacity              Eq. (9)   v_d
  allocate              Alg. 1    MemoryAwareBalancing, then StragglerWorkloadOffloading
  step_times            Eq. (8)   E_f^s, E_b^s of an execution step
  comm_time             Sec. 3.3  E_f^s = E_b^s of a communication step
  plan_hpp              Alg. 2, Eq. (10), Eq. (11)   Q(l, n, p)

(Equation numbers count the paper's displayed equations in order: (1)-(2) in Sec. 2, (3) the
memory model, (4) HPP-Round latency, (5) T_w / T_a, (6) T_e, (7) the allocation target
T(i->j, G), (8) E_f / E_b, (9) capacity, (10) Q update, (11) dominant-step update.)

Readings where the text leaves a choice (each is repeated in the repository's design notes):
  * MOD = 2 * sum(w_l) (parameters and accumulated gradients), OPT = 1 * sum(w_l) (momentum);
    ACT(beta) = beta * sum(act_l).  `act_l` is the activation memory per sample that layer l
    keeps for its backward; `a_l` is the size per sample of its output, which is what crosses a
    stage boundary.  With the paper's one-tensor layers the two are the same number.
  * Every device of a group holds a replica: a group with a member that cannot hold MOD + OPT
    is infeasible.
  * Samples are whole: the proportional shares v_d / sum(v) * beta are rounded by largest
    remainder (ties to the earlier device of the group), so that they add up to beta.
  * The offloading loop moves `block` samples (or what the straggler has left) to the fastest
    device that has memory for them and is not the straggler; a move that does not make the
    slowest device strictly faster is taken back and ends the loop (Eq. (7) asks for the minimum).
  * A communication step moves B * a_j bytes over the slowest link between the two groups.
  * Devices are ordered by memory budget, largest first (ties keep the given order); stage k
    takes the next run of devices in that order (Sec. 3.3, "Dynamic Programming HPP Planning").
  * The head stage of a sub-pipeline of p stages runs K = 2p - 1 warm-up forwards (Sec. 3.2).
  * The dominant step is the first step that maximises M*(E_f+E_b) + sum_{i<s}(E_f^i+E_b^i);
    Eq. (11) compares exactly these aligned totals.

Only tests may import this.  It imports nothing from the HIP package.
"""
import math

INF = math.inf


class Problem:
    """Profiler tables and the resource pool (Sec. 3.3 "DNN Model and Asteroid Profiler").

    tf[d][l][beta], tb[d][l][beta]: FP / BP time of layer l on device d for beta samples,
    beta = 0..B (entry 0 is 0).  a[l], act[l], w[l] in bytes (a, act per sample).  u[d] memory
    budget in bytes.  bw[d][e] bytes per time unit between devices d and e.
    """

    def __init__(self, tf, tb, a, act, w, u, bw, B, M, mod_factor=2.0, opt_factor=1.0, block=1):
        self.tf, self.tb, self.a, self.act, self.w, self.u, self.bw = tf, tb, a, act, w, u, bw
        self.N, self.L, self.B, self.M = len(u), len(a), B, M
        self.mod_factor, self.opt_factor, self.block = mod_factor, opt_factor, block


def stage_memory(pr, lo, hi, K, beta):
    """Eq. (3) for the stage of layers [lo, hi) with K resident micro-batches of beta samples."""
    W = 0.0
    for l in range(lo, hi):
        W += pr.w[l]
    A = 0.0
    for l in range(lo, hi):
        A += pr.act[l]
    return pr.mod_factor * W + pr.opt_factor * W + K * (beta * A)


def max_batch(pr, d, lo, hi, K):
    """Largest beta in 0..B whose Eq. (3) footprint fits u_d; -1 when not even the replica fits."""
    best = -1
    for beta in range(0, pr.B + 1):
        if stage_memory(pr, lo, hi, K, beta) <= pr.u[d]:
            best = beta
    return best


def device_time(pr, d, lo, hi, beta):
    """(sum_l t_f, sum_l t_b) of device d over layers [lo, hi) at batch size beta."""
    f = 0.0
    b = 0.0
    for l in range(lo, hi):
        f += pr.tf[d][l][beta]
        b += pr.tb[d][l][beta]
    return f, b


def capacity(pr, d, lo, hi):
    """Eq. (9): inverse of the FP + BP latency of a whole micro-batch."""
    f, b = device_time(pr, d, lo, hi, pr.B)
    return 1.0 / (f + b)


def proportional_shares(weights, beta):
    """Whole-sample shares of beta in proportion to `weights` (largest remainder)."""
    tot = 0.0
    for x in weights:
        tot += x
    exact = [x / tot * beta for x in weights]
    share = [int(math.floor(e)) for e in exact]
    frac = [e - math.floor(e) for e in exact]
    left = beta - sum(share)
    order = sorted(range(len(weights)), key=lambda k: (-frac[k], k))
    k = 0
    while left > 0:
        share[order[k % len(order)]] += 1
        left -= 1
        k += 1
    k = len(share) - 1
    while left < 0:            # floating point pushed a share over: take it back from the end
        if share[k] > 0:
            share[k] -= 1
            left += 1
        else:
            k -= 1
    return share


def memory_aware_balancing(G, beta, y, room, v):
    """Alg. 1, phase 1.  y and room (samples a device can still take) are updated in place.
    Returns False when the samples cannot be placed."""
    if len(G) == 0 and beta > 0:
        return False
    if beta == 0:
        return True
    share = proportional_shares([v[d] for d in G], beta)
    placed = 0
    for d, s in zip(G, share):
        take = min(s, room[d])
        y[d] += take
        room[d] -= take
        placed += take
    G2 = [d for d in G if room[d] > 0]
    return memory_aware_balancing(G2, beta - placed, y, room, v)


def group_latency(pr, G, lo, hi, y):
    worst = 0.0
    for d in G:
        f, b = device_time(pr, d, lo, hi, y[d])
        worst = max(worst, f + b)
    return worst


def straggler_offloading(pr, G, lo, hi, y, bs):
    """Alg. 1, phase 2."""
    while True:
        t = {}
        for d in G:
            f, b = device_time(pr, d, lo, hi, y[d])
            t[d] = f + b
        order = sorted(G, key=lambda d: (t[d], G.index(d)))
        straggler = order[-1]
        t_old = t[straggler]
        mv = min(pr.block, y[straggler])
        if mv == 0:
            return
        target = None
        for d in order:
            if d != straggler and y[d] + mv <= bs[d]:
                target = d
                break
        if target is None:
            return
        y[straggler] -= mv
        y[target] += mv
        if not group_latency(pr, G, lo, hi, y) < t_old:
            y[straggler] += mv
            y[target] -= mv
            return


def allocate(pr, lo, hi, G, K):
    """Alg. 1 for layers [lo, hi) on device group G (a list of device ids) with K resident
    micro-batches.  Returns {d: y_d} or None when the micro-batch does not fit."""
    bs = {}
    for d in G:
        bs[d] = max_batch(pr, d, lo, hi, K)
        if bs[d] < 0:
            return None
    v = {d: capacity(pr, d, lo, hi) for d in G}
    y = {d: 0 for d in G}
    room = dict(bs)
    if not memory_aware_balancing(list(G), pr.B, y, room, v):
        return None
    straggler_offloading(pr, list(G), lo, hi, y, bs)
    return y


def step_times(pr, lo, hi, G, y):
    """Eq. (8)."""
    Ef = 0.0
    Eb = 0.0
    for d in G:
        f, b = device_time(pr, d, lo, hi, y[d])
        Ef = max(Ef, f)
        Eb = max(Eb, b)
    return Ef, Eb


def allreduce_time(pr, lo, hi, G):
    """Eq. (5), right-hand formula."""
    g = len(G)
    if g <= 1:
        return 0.0
    W = 0.0
    for l in range(lo, hi):
        W += pr.w[l]
    bmin = INF
    for d in G:
        for e in G:
            if d != e:
                bmin = min(bmin, pr.bw[d][e])
    return 2.0 * (g - 1) * W / (g * bmin)


def comm_time(pr, j, G, G2):
    """Time of the communication step behind layer j between groups G and G2 (one direction)."""
    bmin = INF
    for d in G:
        for e in G2:
            bmin = min(bmin, pr.bw[d][e])
    return pr.B * pr.a[j] / bmin


def dominant_step(Ef, Eb, M):
    """Index of the step with the largest aligned FP + BP total (Eq. (11))."""
    best, dm = -1.0, 0
    before = 0.0
    for s in range(len(Ef)):
        val = M * (Ef[s] + Eb[s]) + before
        if val > best:
            best, dm = val, s
        before += Ef[s] + Eb[s]
    return dm


def round_latency(Ef, Eb, Ta, M):
    """Eq. (4) with T_w from Eq. (5) and T_e from Eq. (6).  Ef, Eb, Ta are per step, first
    stage first (execution and communication steps alternate).  Returns (latency, dm)."""
    S = len(Ef)
    dm = dominant_step(Ef, Eb, M)
    worst = 0.0
    for s in range(S):
        Tw = 0.0
        for i in range(0, s):
            Tw += Ef[i]
        Te = M * (Ef[dm] + Eb[dm])
        if s < dm:
            for i in range(s, dm):
                Te += Ef[i] + Eb[i]
        else:
            for i in range(dm, s):
                Te -= Ef[i] + Eb[i]
        worst = max(worst, Tw + Te + Ta[s])
    return worst, dm


def device_order(pr):
    """Devices by memory budget, largest first (stable)."""
    return sorted(range(pr.N), key=lambda d: (-pr.u[d], d))


def evaluate_pipeline(pr, stages):
    """HPP-Round latency of a given configuration.  stages: list of (lo, hi, G) first stage
    first; allocations come from Alg. 1.  Returns (latency, [y dict per stage]) or (inf, None)."""
    P = len(stages)
    Ef, Eb, Ta, ys = [], [], [], []
    for k, (lo, hi, G) in enumerate(stages):
        K = 2 * (P - k) - 1
        y = allocate(pr, lo, hi, G, K)
        if y is None:
            return INF, None
        f, b = step_times(pr, lo, hi, G, y)
        Ef.append(f)
        Eb.append(b)
        Ta.append(allreduce_time(pr, lo, hi, G))
        ys.append(y)
        if k + 1 < P:
            c = comm_time(pr, hi - 1, G, stages[k + 1][2])
            Ef.append(c)
            Eb.append(c)
            Ta.append(0.0)
    return round_latency(Ef, Eb, Ta, pr.M)[0], ys


def plan_hpp(pr):
    """Alg. 2.  Q[(l, n, p)] = (latency, stages) for the last l layers in p stages on the last
    n devices of the memory order.  Returns (latency, stages, allocations) of min_p Q(L, N, p);
    stages as in evaluate_pipeline."""
    L, N = pr.L, pr.N
    order = device_order(pr)
    Q = {}
    for p in range(1, min(L, N) + 1):
        for n in range(1, N + 1):
            for l in range(1, L + 1):
                best = (INF, None)
                for n2 in range(0, n + 1):
                    for l2 in range(0, l + 1):
                        if p == 1:
                            if n2 != 0 or l2 != 0:
                                continue
                            tail = []
                        else:
                            if n2 >= n or l2 >= l:
                                continue
                            sub = Q.get((l2, n2, p - 1))
                            if sub is None or sub[0] == INF:
                                continue
                            tail = sub[1]
                        head = (L - l, L - l2, [order[k] for k in range(N - n, N - n2)])
                        lat, _ = evaluate_pipeline(pr, [head] + tail)
                        if lat < best[0]:
                            best = (lat, [head] + tail)
                Q[(l, n, p)] = best
    best = (INF, None)
    for p in range(1, min(L, N) + 1):
        q = Q[(L, N, p)]
        if q[0] < best[0]:
            best = q
    if best[1] is None:
        return INF, None, None
    lat, ys = evaluate_pipeline(pr, best[1])
    return lat, best[1], ys
