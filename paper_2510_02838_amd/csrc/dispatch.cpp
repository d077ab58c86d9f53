// Resource-Aware Dispatcher: reward weights, communication penalties and an exact solver of
// the dispatch integer program (Section "Resource-Aware Dispatcher", (OBJ), (C0)-(C4);
// Appendix "Dispatch Plan").  Host code only.
//
// Structure used by the solver.  The objective coefficient W_r - Q_{r,i} does not depend on the
// degree k, and a larger k only uses more replicas, so per (request, type) only the smallest
// feasible degree can be part of an optimum that is not matched by one using fewer replicas:
// the program is a multiple-choice knapsack with one capacity per type.  It is solved depth
// first with the Lagrangian bound
//     value so far + sum_i lambda_i * usable_i + sum over open requests of
//                    max(0, max_i (v_{r,i} - lambda_i k_{r,i})),
// where usable_i is the idle count of type i rounded down to what the open requests can use
// (a multiple of the gcd of their degrees on i, zero if below the smallest): degrees are
// powers of two, and without the rounding equal-valued requests that do not divide the
// capacity keep the bound above every incumbent and the search enumerates their subsets.
// States (position in the request order, replicas left per type) already entered with at
// least the same value are not entered again, which makes the search a lazily evaluated
// dynamic program over the states the bound leaves open.
// The multipliers come from a few rounds of per-coordinate bisection on the dual function;
// any lambda >= 0 gives a valid bound, a better one only prunes more.
#include "../../include/dispatch.h"

#include <algorithm>
#include <cmath>
#include <numeric>
#include <unordered_map>
#include <vector>

namespace {

struct Opt { int type, k, kidx; double v; };
struct Item {
  int r, n;
  Opt o[4];
  double best_red;      // max_i (v - lambda_i k), may be negative
  int order[5], n_order;  // option indices in trial order; -1 = leave undispatched
};

// search state: position in the item order and idle replicas left per type
struct StateKey {
  int pos, rem[4];
  bool operator==(const StateKey& o) const {
    return pos == o.pos && rem[0] == o.rem[0] && rem[1] == o.rem[1] && rem[2] == o.rem[2] && rem[3] == o.rem[3];
  }
};
struct StateHash {
  size_t operator()(const StateKey& k) const {
    unsigned long long h = 0x9E3779B97F4A7C15ull * (unsigned)(k.pos + 1);
    for (int i = 0; i < 4; ++i) { h ^= (unsigned)k.rem[i] + 0x9E3779B97F4A7C15ull + (h << 6) + (h >> 2); }
    return (size_t)h;
  }
};

bool finite_all(const double* p, long long n) {
  for (long long i = 0; i < n; ++i)
    if (!std::isfinite(p[i])) return false;
  return true;
}

bool shape_ok(int R, int I, int K) { return R >= 0 && I >= 1 && I <= 4 && K >= 1 && K <= 4; }

}  // namespace

extern "C" int tds_reward_weights(int R, int I, int K, const double* t, const unsigned char* feas,
                                  const double* deadline, double tau, double c_on, double c_late,
                                  double alpha, double* W) {
  if (!shape_ok(R, I, K) || !t || !feas || !deadline || !W) return TDS_EINVAL;
  if (!finite_all(t, (long long)R * I * K) || !finite_all(deadline, R) || !std::isfinite(tau)) return TDS_EINVAL;
  for (int r = 0; r < R; ++r) {
    double best = INFINITY;
    for (int j = 0; j < I * K; ++j)
      if (feas[(size_t)r * I * K + j]) best = std::min(best, tau + t[(size_t)r * I * K + j]);
    if (!std::isfinite(best)) { W[r] = 0.0; continue; }
    if (best <= deadline[r]) { W[r] = c_on; continue; }
    const double scale = std::max(1.0, best / deadline[r]);
    W[r] = c_late * std::max(1.0, scale - alpha + 1.0);
  }
  return TDS_OK;
}

extern "C" int tds_comm_penalty(int R, int I, const double* length, const double* beta, double* Q) {
  if (R < 0 || I < 1 || I > 4 || !length || !beta || !Q) return TDS_EINVAL;
  for (int r = 0; r < R; ++r)
    for (int i = 0; i < I; ++i) Q[(size_t)r * I + i] = beta[i] * length[r];
  return TDS_OK;
}

extern "C" int tds_dispatch_solve(int R, int I, int K, const int* degrees, const double* W, const double* Q,
                                  const unsigned char* feas, const int* B, const double* t,
                                  const double* deadline, double tau, long long node_limit, double gap_abs,
                                  int* choice_type, int* choice_degree, unsigned char* D, double* objective,
                                  double* upper_bound, long long* nodes) {
  if (!shape_ok(R, I, K) || !degrees || !W || !Q || !feas || !B || !t || !deadline || !choice_type ||
      !choice_degree || !D || !objective || !upper_bound || !nodes)
    return TDS_EINVAL;
  for (int k = 0; k < K; ++k)
    if (degrees[k] <= 0 || (k && degrees[k] <= degrees[k - 1])) return TDS_EINVAL;
  for (int i = 0; i < I; ++i)
    if (B[i] < 0) return TDS_EINVAL;
  if (!finite_all(W, R) || !finite_all(Q, (long long)R * I) || !finite_all(t, (long long)R * I * K) ||
      !finite_all(deadline, R) || !std::isfinite(tau) || !(gap_abs >= 0.0))
    return TDS_EINVAL;

  // ---- options after dominance: per (r, i) the smallest feasible degree, positive value only
  std::vector<Item> items;
  items.reserve(R);
  for (int r = 0; r < R; ++r) {
    Item it;
    it.r = r; it.n = 0;
    for (int i = 0; i < I; ++i) {
      const double v = W[r] - Q[(size_t)r * I + i];
      if (!(v > 0.0)) continue;
      for (int k = 0; k < K; ++k)
        if (feas[((size_t)r * I + i) * K + k]) {
          if (degrees[k] <= B[i]) it.o[it.n++] = Opt{i, degrees[k], k, v};
          break;
        }
    }
    if (it.n) items.push_back(it);
  }
  const int n = (int)items.size();

  // ---- multipliers.  Start: per-coordinate bisection for the smallest lambda_i whose usage
  // fits B_i (exact for one binding type; with several it can stall at a kink of the dual
  // function).  Then subgradient steps of Polyak length towards a greedy primal value, keeping
  // the multipliers of the lowest dual value seen.
  double lam[4] = {0, 0, 0, 0};
  double vmax = 0.0, greedy_value = 0.0;
  std::vector<int> greedy_type(R, -1);   // type the greedy pass gave request r, or -1
  for (const Item& it : items)
    for (int j = 0; j < it.n; ++j) vmax = std::max(vmax, it.o[j].v);
  // dual value at lam and the replicas its maximiser uses per type
  auto dual = [&](long long use[4]) {
    double L = 0.0;
    for (int i = 0; i < 4; ++i) use[i] = 0;
    for (int i = 0; i < I; ++i) L += lam[i] * B[i];
    for (const Item& it : items) {
      int arg = -1; double best = 0.0;
      for (int j = 0; j < it.n; ++j) {
        const double red = it.o[j].v - lam[it.o[j].type] * it.o[j].k;
        if (red > best) { best = red; arg = j; }
      }
      if (arg >= 0) { L += best; use[it.o[arg].type] += it.o[arg].k; }
    }
    return L;
  };
  long long use[4];
  for (int round = 0; round < 4; ++round)
    for (int i = 0; i < I; ++i) {
      lam[i] = 0.0;
      dual(use);
      if (use[i] <= B[i]) continue;
      double lo = 0.0, hi = vmax;      // usage(hi) = 0 <= B_i
      for (int s = 0; s < 40; ++s) {
        lam[i] = 0.5 * (lo + hi);
        dual(use);
        if (use[i] <= B[i]) hi = lam[i]; else lo = lam[i];
      }
      lam[i] = hi;
    }
  {
    // greedy primal value: requests by value per replica, each to its best option that still fits
    std::vector<int> ord(items.size());
    std::iota(ord.begin(), ord.end(), 0);
    auto dens = [&](const Item& it) {
      double d = 0.0;
      for (int j = 0; j < it.n; ++j) d = std::max(d, it.o[j].v / it.o[j].k);
      return d;
    };
    std::vector<double> dn(items.size());
    for (size_t q = 0; q < items.size(); ++q) dn[q] = dens(items[q]);
    std::stable_sort(ord.begin(), ord.end(), [&](int a, int b) { return dn[a] > dn[b]; });
    int left[4] = {0, 0, 0, 0};
    for (int i = 0; i < I; ++i) left[i] = B[i];
    double target = 0.0;
    for (int q : ord) {
      int arg = -1;
      for (int j = 0; j < items[q].n; ++j)
        if (items[q].o[j].k <= left[items[q].o[j].type] && (arg < 0 || items[q].o[j].v > items[q].o[arg].v)) arg = j;
      if (arg >= 0) {
        left[items[q].o[arg].type] -= items[q].o[arg].k; target += items[q].o[arg].v;
        greedy_type[items[q].r] = items[q].o[arg].type;
      }
    }
    greedy_value = target;
    double best_L = dual(use), best_lam[4] = {lam[0], lam[1], lam[2], lam[3]}, theta = 1.0;
    int stale = 0;
    for (int iter = 0; iter < 4000 && best_L - target > 1e-9; ++iter) {
      const double L = dual(use);
      if (L < best_L - 1e-12) { best_L = L; for (int i = 0; i < 4; ++i) best_lam[i] = lam[i]; stale = 0; }
      else if (++stale >= 40) { theta *= 0.5; stale = 0; for (int i = 0; i < 4; ++i) lam[i] = best_lam[i]; }
      double g2 = 0.0, g[4] = {0, 0, 0, 0};
      for (int i = 0; i < I; ++i) {
        g[i] = (double)B[i] - (double)use[i];
        if (lam[i] <= 0.0 && g[i] > 0.0) g[i] = 0.0;       // projected: cannot go below zero
        g2 += g[i] * g[i];
      }
      if (g2 == 0.0 || theta < 1e-6) break;
      const double step = theta * (L - target) / g2;
      for (int i = 0; i < I; ++i) lam[i] = std::max(0.0, lam[i] - step * g[i]);
    }
    for (int i = 0; i < 4; ++i) lam[i] = best_lam[i];
  }

  // ---- trial order: strongest reduced profit first; inside an item best reduced option first
  for (Item& it : items) {
    int idx[4] = {0, 1, 2, 3};
    std::sort(idx, idx + it.n, [&](int a, int b) {
      const double ra = it.o[a].v - lam[it.o[a].type] * it.o[a].k, rb = it.o[b].v - lam[it.o[b].type] * it.o[b].k;
      if (ra != rb) return ra > rb;
      return it.o[a].k < it.o[b].k;
    });
    it.best_red = it.o[idx[0]].v - lam[it.o[idx[0]].type] * it.o[idx[0]].k;
    // options the multipliers price as worth their replicas, then "leave", then the rest
    it.n_order = 0;
    bool left = false;
    for (int j = 0; j < it.n; ++j) {
      const double red = it.o[idx[j]].v - lam[it.o[idx[j]].type] * it.o[idx[j]].k;
      if (!left && red <= 0.0) { it.order[it.n_order++] = -1; left = true; }
      it.order[it.n_order++] = idx[j];
    }
    if (!left) it.order[it.n_order++] = -1;
  }
  std::stable_sort(items.begin(), items.end(), [](const Item& a, const Item& b) { return a.best_red > b.best_red; });

  std::vector<double> suffix(n + 1, 0.0);
  std::vector<int> min_k((size_t)(n + 1) * 4, 0), gcd_k((size_t)(n + 1) * 4, 0);   // 0 = no open option on the type
  for (int p = n - 1; p >= 0; --p) {
    suffix[p] = suffix[p + 1] + std::max(0.0, items[p].best_red);
    for (int i = 0; i < 4; ++i) { min_k[p * 4 + i] = min_k[(p + 1) * 4 + i]; gcd_k[p * 4 + i] = gcd_k[(p + 1) * 4 + i]; }
    for (int j = 0; j < items[p].n; ++j) {
      const int i = items[p].o[j].type, k = items[p].o[j].k;
      min_k[p * 4 + i] = min_k[p * 4 + i] ? std::min(min_k[p * 4 + i], k) : k;
      gcd_k[p * 4 + i] = std::gcd(gcd_k[p * 4 + i], k);
    }
  }
  int rem[4] = {0, 0, 0, 0};
  for (int i = 0; i < I; ++i) rem[i] = B[i];
  auto bound_at = [&](int p, double value) {
    double b = value + suffix[p];
    for (int i = 0; i < I; ++i) {
      const int mk = min_k[p * 4 + i], g = gcd_k[p * 4 + i];
      if (!mk || rem[i] < mk) continue;
      b += lam[i] * (double)(rem[i] / g * g);
    }
    return b;
  };
  const double root_bound = bound_at(0, 0.0);

  // ---- depth-first search
  std::vector<int> cur(n + 1, 0), taken(n, -1), best_taken(n, -1);
  double value = 0.0, best = -1.0;
  if (greedy_value > 0.0) {               // the greedy assignment is the first incumbent
    best = greedy_value;
    for (int q = 0; q < n; ++q)
      for (int j = 0; j < items[q].n; ++j)
        if (items[q].o[j].type == greedy_type[items[q].r]) best_taken[q] = j;
  }
  {
    // Second incumbent, guided by the multipliers: in search order, every request takes its
    // best option that the multipliers price as worth its replicas and that still fits; what
    // is left of the capacity is then handed out in the same order to whatever fits.
    std::vector<int> pick(n, -1);
    int left[4] = {0, 0, 0, 0};
    for (int i = 0; i < I; ++i) left[i] = B[i];
    double val = 0.0;
    for (int pass = 0; pass < 2; ++pass)
      for (int q = 0; q < n; ++q) {
        if (pick[q] >= 0) continue;
        const Item& it = items[q];
        for (int e = 0; e < it.n_order; ++e) {
          const int c = it.order[e];
          if (c < 0) { if (pass == 0) break; else continue; }
          if (it.o[c].k <= left[it.o[c].type]) { left[it.o[c].type] -= it.o[c].k; val += it.o[c].v; pick[q] = c; break; }
        }
      }
    if (val > best) { best = val; best_taken = pick; }
  }
  long long visited = 0;
  bool limit_hit = false, gap_stop = false;
  const double eps = 1e-9;
  // Dominance: a state (position, replicas left) entered before with at least this value has
  // had its whole subtree searched (or cut against an incumbent no worse than today's), so a
  // second entry cannot find anything better.  Requests with near-equal rewards reach the same
  // state along many paths; the bound alone cannot separate them.
  std::unordered_map<StateKey, double, StateHash> seen;
  const size_t seen_cap = (size_t)4 << 20;
  int p = 0;
  // cur[p]: next entry of items[p].order to try; entering a node = cur[p] == 0
  while (p >= 0) {
    if (p == n) {
      if (value > best) {
        best = value; best_taken = taken;
        if (root_bound - best <= gap_abs) { gap_stop = true; break; }
      }
      --p;
      continue;
    }
    Item& it = items[p];
    if (cur[p] == 0) {
      ++visited;
      if (node_limit > 0 && visited > node_limit) { limit_hit = true; break; }
      if (bound_at(p, value) <= best + eps) { --p; continue; }
      const StateKey key{p, {rem[0], rem[1], rem[2], rem[3]}};
      auto f = seen.find(key);
      if (f != seen.end()) {
        if (value <= f->second + eps) { --p; continue; }
        f->second = value;
      } else if (seen.size() < seen_cap) {
        seen.emplace(key, value);
      }
    } else {
      // undo the option tried last
      const int last = it.order[cur[p] - 1];
      if (last >= 0 && taken[p] == last) { rem[it.o[last].type] += it.o[last].k; value -= it.o[last].v; taken[p] = -1; }
    }
    bool moved = false;
    while (cur[p] < it.n_order) {
      const int c = it.order[cur[p]++];
      if (c < 0) { taken[p] = -1; moved = true; break; }
      if (it.o[c].k <= rem[it.o[c].type]) {
        rem[it.o[c].type] -= it.o[c].k; value += it.o[c].v; taken[p] = c; moved = true;
        break;
      }
    }
    if (!moved) { cur[p] = 0; --p; continue; }
    ++p;
    cur[p] = 0;
  }
  if (best < 0.0) { best = 0.0; std::fill(best_taken.begin(), best_taken.end(), -1); }   // limit before any leaf

  for (int r = 0; r < R; ++r) { choice_type[r] = -1; choice_degree[r] = -1; D[r] = 0; }
  double obj = 0.0;
  for (int q = 0; q < n; ++q) {
    const int c = best_taken[q];
    if (c < 0) continue;
    const Item& it = items[q];
    const Opt& o = it.o[c];
    choice_type[it.r] = o.type; choice_degree[it.r] = o.k;
    obj += o.v;
    D[it.r] = tau + t[((size_t)it.r * I + o.type) * K + o.kidx] <= deadline[it.r] ? 1 : 0;
  }
  *objective = obj;
  *upper_bound = (limit_hit || gap_stop) ? std::max(root_bound, obj) : obj;
  *nodes = visited;
  return limit_hit ? TDS_LIMIT : TDS_OK;
}
