// Parallelism planner (Sec. 3.3): Eq. (3)-(11), Alg. 1 and Alg. 2 on the host.
//
// Layer sums come from prefix sums over layers (per device and batch size), so a stage's
// E_f / E_b / memory cost O(1); the dynamic programme keeps per state Q(l, n, p) the step
// times of its pipeline and its dominant step, so that prepending a stage costs O(p) and not
// a re-evaluation of the tail.
#include <algorithm>
#include <cmath>
#include <limits>
#include <numeric>
#include <string>
#include <vector>

#include "../../include/asteroid_planner.h"

namespace ast {
void set_last_error(const std::string& msg);  // api.cpp
}

namespace {

constexpr double INF = std::numeric_limits<double>::infinity();

int32_t fail(const std::string& msg) {
  ast::set_last_error(msg);
  return AST_EINVAL;
}

struct Tables {
  const ast_plan_problem* pr;
  int L, N, B;
  std::vector<double> pf, pb;  // [N][B+1][L+1] prefix sums over layers of t_f, t_b
  std::vector<double> pw, pact, pfix;  // [L+1]

  explicit Tables(const ast_plan_problem* p) : pr(p), L(p->L), N(p->N), B(p->B) {
    const size_t row = (size_t)L + 1;
    pf.assign((size_t)N * (B + 1) * row, 0.0);
    pb.assign((size_t)N * (B + 1) * row, 0.0);
    for (int d = 0; d < N; ++d)
      for (int b = 0; b <= B; ++b) {
        double* f = &pf[((size_t)d * (B + 1) + b) * row];
        double* g = &pb[((size_t)d * (B + 1) + b) * row];
        for (int l = 0; l < L; ++l) {
          const size_t src = ((size_t)d * L + l) * (B + 1) + b;
          f[l + 1] = f[l] + p->host_tf[src];
          g[l + 1] = g[l] + p->host_tb[src];
        }
      }
    pw.assign(row, 0.0);
    pact.assign(row, 0.0);
    pfix.assign(row, 0.0);
    for (int l = 0; l < L; ++l) {
      pw[l + 1] = pw[l] + p->host_w[l];
      pact[l + 1] = pact[l] + p->host_act[l];
      pfix[l + 1] = pfix[l] + (p->host_fixed ? p->host_fixed[l] : 0.0);
    }
  }
  double tf(int d, int lo, int hi, int beta) const {
    const double* f = &pf[((size_t)d * (B + 1) + beta) * (L + 1)];
    return f[hi] - f[lo];
  }
  double tb(int d, int lo, int hi, int beta) const {
    const double* g = &pb[((size_t)d * (B + 1) + beta) * (L + 1)];
    return g[hi] - g[lo];
  }
  double weights(int lo, int hi) const { return pw[hi] - pw[lo]; }
  // Eq. (3)
  double memory(int lo, int hi, int K, int beta) const {
    const double W = weights(lo, hi), A = pact[hi] - pact[lo];
    return pr->mod_factor * W + pr->opt_factor * W + K * (beta * A) + (pfix[hi] - pfix[lo]);
  }
  // largest beta in 0..B that fits the budget of d; -1 when the replica alone does not
  int max_batch(int d, int lo, int hi, int K) const {
    const double u = pr->host_u[d];
    if (!(memory(lo, hi, K, 0) <= u)) return -1;
    int a = 0, b = B;  // memory is non-decreasing in beta: bisect
    while (a < b) {
      const int m = (a + b + 1) / 2;
      if (memory(lo, hi, K, m) <= u) a = m; else b = m - 1;
    }
    return a;
  }
  double bw(int d, int e) const { return pr->host_bw[(size_t)d * N + e]; }
};

// whole-sample shares of beta in proportion to v (largest remainder, ties to the earlier entry)
void proportional_shares(const std::vector<double>& v, int beta, std::vector<int>& share) {
  const int g = (int)v.size();
  double tot = 0.0;
  for (double x : v) tot += x;
  std::vector<double> frac(g);
  share.assign(g, 0);
  int given = 0;
  for (int k = 0; k < g; ++k) {
    const double e = v[k] / tot * beta;
    const double fl = std::floor(e);
    share[k] = (int)fl;
    frac[k] = e - fl;
    given += share[k];
  }
  std::vector<int> order(g);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int x, int y) { return frac[x] > frac[y]; });
  int left = beta - given;
  for (int k = 0; left > 0; ++k, --left) share[order[k % g]] += 1;
  for (int k = g - 1; left < 0;) {
    if (share[k] > 0) { share[k] -= 1; ++left; } else { --k; }
  }
}

struct Alloc {
  std::vector<int> y;  // per member of the group
  double Ef = 0, Eb = 0;
};

// Alg. 1 on devices G (ids) for layers [lo, hi) with K resident micro-batches
bool allocate(const Tables& t, int lo, int hi, const int* G, int g, int K, Alloc& out) {
  const int B = t.B, block = t.pr->block;
  std::vector<int> bs(g), room(g);
  std::vector<double> v(g);
  for (int k = 0; k < g; ++k) {
    bs[k] = t.max_batch(G[k], lo, hi, K);
    if (bs[k] < 0) return false;
    room[k] = bs[k];
    v[k] = 1.0 / (t.tf(G[k], lo, hi, B) + t.tb(G[k], lo, hi, B));  // Eq. (9)
  }
  std::vector<int>& y = out.y;
  y.assign(g, 0);
  // phase 1: the recursion of MemoryAwareBalancing as a loop over shrinking member lists
  std::vector<int> members(g);
  std::iota(members.begin(), members.end(), 0);
  int beta = B;
  std::vector<double> vv;
  std::vector<int> share;
  while (beta > 0) {
    if (members.empty()) return false;
    vv.clear();
    for (int k : members) vv.push_back(v[k]);
    proportional_shares(vv, beta, share);
    int placed = 0;
    for (size_t i = 0; i < members.size(); ++i) {
      const int k = members[i];
      const int take = std::min(share[i], room[k]);
      y[k] += take;
      room[k] -= take;
      placed += take;
    }
    std::vector<int> next;
    for (int k : members)
      if (room[k] > 0) next.push_back(k);
    members.swap(next);
    beta -= placed;
  }
  // phase 2: StragglerWorkloadOffloading
  std::vector<double> time(g);
  std::vector<int> order(g);
  for (;;) {
    for (int k = 0; k < g; ++k) time[k] = t.tf(G[k], lo, hi, y[k]) + t.tb(G[k], lo, hi, y[k]);
    std::iota(order.begin(), order.end(), 0);
    std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return time[a] < time[b]; });
    const int straggler = order[g - 1];
    const double t_old = time[straggler];
    const int mv = std::min(block, y[straggler]);
    if (mv == 0) break;
    int target = -1;
    for (int k : order)
      if (k != straggler && y[k] + mv <= bs[k]) { target = k; break; }
    if (target < 0) break;
    y[straggler] -= mv;
    y[target] += mv;
    double worst = 0.0;
    for (int k = 0; k < g; ++k) {
      const double tk = (k == straggler || k == target) ? t.tf(G[k], lo, hi, y[k]) + t.tb(G[k], lo, hi, y[k]) : time[k];
      worst = std::max(worst, tk);
    }
    if (!(worst < t_old)) {
      y[straggler] += mv;
      y[target] -= mv;
      break;
    }
  }
  out.Ef = out.Eb = 0.0;  // Eq. (8)
  for (int k = 0; k < g; ++k) {
    out.Ef = std::max(out.Ef, t.tf(G[k], lo, hi, y[k]));
    out.Eb = std::max(out.Eb, t.tb(G[k], lo, hi, y[k]));
  }
  return true;
}

// Eq. (5), right-hand formula
double allreduce_time(const Tables& t, int lo, int hi, const int* G, int g) {
  if (g <= 1) return 0.0;
  double bmin = INF;
  for (int i = 0; i < g; ++i)
    for (int j = 0; j < g; ++j)
      if (i != j) bmin = std::min(bmin, t.bw(G[i], G[j]));
  return 2.0 * (g - 1) * t.weights(lo, hi) / (g * bmin);
}

// one direction of the communication step behind layer j between two groups
double comm_time(const Tables& t, int j, const int* G, int g, const int* G2, int g2) {
  double bmin = INF;
  for (int i = 0; i < g; ++i)
    for (int k = 0; k < g2; ++k) bmin = std::min(bmin, t.bw(G[i], G2[k]));
  return t.B * t.pr->host_a[j] / bmin;
}

// Eq. (4) with T_w (Eq. (5)) and T_e (Eq. (6)) for a known dominant step
double latency_given_dm(const double* Ef, const double* Eb, const double* Ta, int S, int M, int dm) {
  double worst = 0.0;
  for (int s = 0; s < S; ++s) {
    double Tw = 0.0;
    for (int i = 0; i < s; ++i) Tw += Ef[i];
    double Te = M * (Ef[dm] + Eb[dm]);
    if (s < dm)
      for (int i = s; i < dm; ++i) Te += Ef[i] + Eb[i];
    else
      for (int i = dm; i < s; ++i) Te -= Ef[i] + Eb[i];
    worst = std::max(worst, Tw + Te + Ta[s]);
  }
  return worst;
}

int dominant_step(const double* Ef, const double* Eb, int S, int M) {
  double best = -1.0, before = 0.0;
  int dm = 0;
  for (int s = 0; s < S; ++s) {
    const double val = M * (Ef[s] + Eb[s]) + before;
    if (val > best) { best = val; dm = s; }
    before += Ef[s] + Eb[s];
  }
  return dm;
}

bool check_problem(const ast_plan_problem* pr) {
  if (!pr) return false;
  if (pr->L < 1 || pr->N < 1 || pr->B < 1 || pr->M < 1 || pr->block < 1) return false;
  if (!pr->host_tf || !pr->host_tb || !pr->host_a || !pr->host_act || !pr->host_w || !pr->host_u || !pr->host_bw)
    return false;
  if (!(pr->mod_factor >= 0) || !(pr->opt_factor >= 0)) return false;
  return true;
}

// state of Q(l, n, p): steps of the pipeline (head first), dominant step, back-pointer
struct State {
  double lat = INF;
  int l2 = 0, n2 = 0, dm = 0;
  std::vector<double> Ef, Eb, Ta;
};

}  // namespace

extern "C" {

int32_t asteroid_plan_stage_memory(const ast_plan_problem* pr, int32_t lo, int32_t hi, int32_t K, int32_t beta,
                                   double* bytes) {
  if (!check_problem(pr) || !bytes) return fail("plan_stage_memory: bad problem or NULL output");
  if (lo < 0 || hi > pr->L || lo >= hi || K < 1 || beta < 0 || beta > pr->B)
    return fail("plan_stage_memory: layer range, K or beta out of range");
  double W = 0.0, A = 0.0;
  for (int l = lo; l < hi; ++l) W += pr->host_w[l];
  for (int l = lo; l < hi; ++l) A += pr->host_act[l];
  double F = 0.0;
  if (pr->host_fixed)
    for (int l = lo; l < hi; ++l) F += pr->host_fixed[l];
  *bytes = pr->mod_factor * W + pr->opt_factor * W + K * (beta * A) + F;
  return AST_OK;
}

int32_t asteroid_plan_allocate(const ast_plan_problem* pr, int32_t lo, int32_t hi, const int32_t* host_group,
                               int32_t g, int32_t K, int32_t* host_y, double* Ef, double* Eb, int32_t* feasible) {
  if (!check_problem(pr) || !host_group || !host_y || !Ef || !Eb || !feasible)
    return fail("plan_allocate: bad problem or NULL argument");
  if (lo < 0 || hi > pr->L || lo >= hi || K < 1 || g < 1 || g > pr->N)
    return fail("plan_allocate: layer range, K or group size out of range");
  std::vector<char> seen(pr->N, 0);
  for (int k = 0; k < g; ++k) {
    if (host_group[k] < 0 || host_group[k] >= pr->N || seen[host_group[k]])
      return fail("plan_allocate: device ids must be distinct and in 0..N-1");
    seen[host_group[k]] = 1;
  }
  const Tables t(pr);
  Alloc a;
  std::vector<int> G(host_group, host_group + g);
  if (!allocate(t, lo, hi, G.data(), g, K, a)) {
    *feasible = 0;
    return AST_OK;
  }
  for (int k = 0; k < g; ++k) host_y[k] = a.y[k];
  *Ef = a.Ef;
  *Eb = a.Eb;
  *feasible = 1;
  return AST_OK;
}

int32_t asteroid_plan_round_latency(int32_t S, const double* host_Ef, const double* host_Eb, const double* host_Ta,
                                    int32_t M, double* latency, int32_t* dm) {
  if (S < 1 || (S & 1) == 0 || M < 1 || !host_Ef || !host_Eb || !host_Ta || !latency || !dm)
    return fail("plan_round_latency: S must be odd and positive, M positive, pointers non-NULL");
  const int d = dominant_step(host_Ef, host_Eb, S, M);
  *dm = d;
  *latency = latency_given_dm(host_Ef, host_Eb, host_Ta, S, M, d);
  return AST_OK;
}

int32_t asteroid_plan_hpp(const ast_plan_problem* pr, int32_t* P, int32_t* host_stage_lo, int32_t* host_stage_ndev,
                          int32_t* host_dev_order, int32_t* host_y, double* latency) {
  if (!check_problem(pr) || !P || !host_stage_lo || !host_stage_ndev || !host_dev_order || !host_y || !latency)
    return fail("plan_hpp: bad problem or NULL argument");
  const int L = pr->L, N = pr->N, M = pr->M;
  const Tables t(pr);
  std::vector<int> order(N);
  std::iota(order.begin(), order.end(), 0);
  std::stable_sort(order.begin(), order.end(), [&](int a, int b) { return pr->host_u[a] > pr->host_u[b]; });

  const int Pmax = std::min(L, N);
  // Q[p][n][l]; index 0 unused
  std::vector<State> Q((size_t)(Pmax + 1) * (N + 1) * (L + 1));
  auto at = [&](int p, int n, int l) -> State& { return Q[((size_t)p * (N + 1) + n) * (L + 1) + l]; };
  Alloc a;
  std::vector<double> Ef, Eb, Ta;
  for (int p = 1; p <= Pmax; ++p) {
    const int S = 2 * p - 1, K = 2 * p - 1;
    Ef.assign(S, 0.0);
    Eb.assign(S, 0.0);
    Ta.assign(S, 0.0);
    for (int n = 1; n <= N; ++n)
      for (int l = 1; l <= L; ++l) {
        State& best = at(p, n, l);
        const int n2_lo = p == 1 ? 0 : p - 1, n2_hi = p == 1 ? 0 : n - 1;
        const int l2_lo = p == 1 ? 0 : p - 1, l2_hi = p == 1 ? 0 : l - 1;
        for (int n2 = n2_lo; n2 <= n2_hi; ++n2)
          for (int l2 = l2_lo; l2 <= l2_hi; ++l2) {
            const State* sub = nullptr;
            if (p > 1) {
              sub = &at(p - 1, n2, l2);
              if (sub->lat == INF) continue;
            }
            // the new execution step: layers [L-l, L-l2) on devices order[N-n .. N-n2)
            const int lo = L - l, hi = L - l2, g = n - n2;
            const int* G = &order[N - n];
            if (!allocate(t, lo, hi, G, g, K, a)) continue;
            Ef[0] = a.Ef;
            Eb[0] = a.Eb;
            Ta[0] = allreduce_time(t, lo, hi, G, g);
            int dm = 0;
            if (p > 1) {
              // the new communication step, then the steps of the sub-pipeline
              const State& head_of_sub = *sub;
              const int g2 = n2 - at(p - 1, n2, l2).n2;
              const double c = comm_time(t, hi - 1, G, g, &order[N - n2], g2);
              Ef[1] = Eb[1] = c;
              Ta[1] = 0.0;
              std::copy(head_of_sub.Ef.begin(), head_of_sub.Ef.end(), Ef.begin() + 2);
              std::copy(head_of_sub.Eb.begin(), head_of_sub.Eb.end(), Eb.begin() + 2);
              std::copy(head_of_sub.Ta.begin(), head_of_sub.Ta.end(), Ta.begin() + 2);
              // Eq. (11): aligned totals of the new execution step, the new communication
              // step and the sub-pipeline's dominant step; the first of the largest wins
              const double v_ne = M * (Ef[0] + Eb[0]);
              const double v_nc = M * (Ef[1] + Eb[1]) + (Ef[0] + Eb[0]);
              const int old = sub->dm + 2;
              double before = 0.0;
              for (int i = 0; i < old; ++i) before += Ef[i] + Eb[i];
              const double v_old = M * (Ef[old] + Eb[old]) + before;
              double vbest = v_ne;
              if (v_nc > vbest) { vbest = v_nc; dm = 1; }
              if (v_old > vbest) { vbest = v_old; dm = old; }
            }
            const double lat = latency_given_dm(Ef.data(), Eb.data(), Ta.data(), S, M, dm);
            if (lat < best.lat) {
              best.lat = lat;
              best.l2 = l2;
              best.n2 = n2;
              best.dm = dm;
              best.Ef = Ef;
              best.Eb = Eb;
              best.Ta = Ta;
            }
          }
      }
  }
  int bp = 0;
  double blat = INF;
  for (int p = 1; p <= Pmax; ++p)
    if (at(p, N, L).lat < blat) { blat = at(p, N, L).lat; bp = p; }
  for (int d = 0; d < N; ++d) {
    host_dev_order[d] = order[d];
    host_y[d] = 0;
    host_stage_ndev[d] = 0;
  }
  for (int k = 0; k <= N; ++k) host_stage_lo[k] = L;
  *P = bp;
  *latency = blat;
  if (bp == 0) return AST_OK;
  int l = L, n = N;
  for (int k = 0, p = bp; p >= 1; ++k, --p) {
    const State& s = at(p, n, l);
    const int lo = L - l, hi = L - s.l2, g = n - s.n2;
    host_stage_lo[k] = lo;
    host_stage_ndev[k] = g;
    if (!allocate(t, lo, hi, &order[N - n], g, 2 * p - 1, a)) return fail("plan_hpp: internal: stage no longer feasible");
    for (int i = 0; i < g; ++i) host_y[order[N - n + i]] = a.y[i];
    l = s.l2;
    n = s.n2;
  }
  host_stage_lo[bp] = L;
  return AST_OK;
}

}  // extern "C"
