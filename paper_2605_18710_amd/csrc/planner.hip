// Host-side planning for one GPU: the interference correction of the performance model
// (Sec. 3.3, Eq. 7-8), the per-stage allocation problem StageEval (Sec. 3.1, Eq. 4-5;
// Sec. 3.4: binary search on a target latency with a feasibility test per trial) and the
// greedy stage formation of Alg. 1 with early pruning and result caching (Sec. 3.4).
//
// On one GPU a stage of at most 16 modules over at most 16 quota levels is small enough for
// exact feasibility tests by depth-first enumeration, which stands where the paper calls a
// constraint solver; the optimum found is the same.  No GPU call is made in this file.
#include <math.h>
#include <string.h>
#include <algorithm>
#include <limits>
#include <map>
#include <vector>
#include "common.h"

namespace {

constexpr int kMaxModules = 16, kMaxPoints = 16;
const double kInf = std::numeric_limits<double>::infinity();

// Eq. 8 on one GPU: e1 + e2 * sum B + e3 * prod B over the modules placed on it.
double delta_of(const double* e, int k, const double* bw) {
  double s = 0.0, p = 1.0;
  for (int i = 0; i < k; ++i) { s += bw[i]; p *= bw[i]; }
  return e[0] + e[1] * s + e[2] * p;
}

// Solves the n x n normal equations A x = b (n <= 3) by Gaussian elimination with partial
// pivoting; false when a pivot vanishes relative to the matrix scale.
bool solve_small(int n, double A[3][3], double* b, double* x) {
  double scale = 0.0;
  for (int i = 0; i < n; ++i) for (int j = 0; j < n; ++j) scale = std::max(scale, fabs(A[i][j]));
  if (scale == 0.0) return false;
  for (int c = 0; c < n; ++c) {
    int piv = c;
    for (int r = c + 1; r < n; ++r) if (fabs(A[r][c]) > fabs(A[piv][c])) piv = r;
    if (fabs(A[piv][c]) <= 1e-13 * scale) return false;
    if (piv != c) { for (int j = 0; j < n; ++j) std::swap(A[piv][j], A[c][j]); std::swap(b[piv], b[c]); }
    for (int r = c + 1; r < n; ++r) {
      const double f = A[r][c] / A[c][c];
      for (int j = c; j < n; ++j) A[r][j] -= f * A[c][j];
      b[r] -= f * b[c];
    }
  }
  for (int r = n - 1; r >= 0; --r) {
    double v = b[r];
    for (int j = r + 1; j < n; ++j) v -= A[r][j] * x[j];
    x[r] = v / A[r][r];
  }
  return true;
}

struct Problem {
  int n, np, total;
  std::vector<int> cus;                 // [np]
  std::vector<double> t, bw;            // [n*np]
  bool rect;
  int form;
  double e[3];
  std::vector<std::pair<int, int>> edges;
};

struct Eval { double t; int level[kMaxModules]; };   // level[m] = grid index, -1 for non-members

// StageEval without interference terms: the objective is separable, so a trial latency tau
// is feasible exactly when every module has a level with time <= tau and the cheapest such
// levels fit the CU budget together.  Binary search over the sorted distinct times; the
// smallest feasible one is the stage time.  Then the lexicographically smallest level
// tuple that attains it is recovered by a depth-first walk.
struct StageSolver {
  const Problem& P;
  std::vector<int> mods;
  explicit StageSolver(const Problem& p, uint32_t mask) : P(p) {
    for (int m = 0; m < p.n; ++m) if (mask >> m & 1) mods.push_back(m);
  }
  double T(int m, int p) const { return P.t[(size_t)m * P.np + p]; }

  bool feasible_separable(double tau) const {
    long need = 0;
    for (int m : mods) {
      int best = -1;
      for (int p = 0; p < P.np; ++p)
        if (T(m, p) <= tau && (best < 0 || P.cus[p] < P.cus[best])) best = p;
      if (best < 0) return false;
      need += P.cus[best];
    }
    return need <= P.total;
  }

  // first (lexicographic) level tuple with stage time <= tau under the budget
  bool first_tuple(size_t k, long used, double tau, int* lv) const {
    if (k == mods.size()) return true;
    // cheapest completion of the remaining modules, to cut branches that cannot fit
    for (int p = 0; p < P.np; ++p) {
      if (T(mods[k], p) > tau || used + P.cus[p] > P.total) continue;
      lv[k] = p;
      if (first_tuple(k + 1, used + P.cus[p], tau, lv)) return true;
    }
    return false;
  }

  // With interference terms the delay couples the modules: every level tuple within the
  // budget is visited, in lexicographic order, and the first minimum is kept.
  void walk_rectified(size_t k, long used, int* lv, Eval* best) const {
    if (k == mods.size()) {
      double b[kMaxModules];
      for (size_t i = 0; i < mods.size(); ++i) b[i] = P.bw[(size_t)mods[i] * P.np + lv[i]];
      double t = -kInf;
      if (P.form == MOSAIC_DELAY_ABSOLUTE) {
        const double d = delta_of(P.e, (int)mods.size(), b);
        for (size_t i = 0; i < mods.size(); ++i) t = std::max(t, T(mods[i], lv[i]) + d);
      } else {
        // the expression over the other modules of the stage, charged as a fraction of own time
        double peers[kMaxModules];
        for (size_t i = 0; i < mods.size(); ++i) {
          int k = 0;
          for (size_t j = 0; j < mods.size(); ++j) if (j != i) peers[k++] = b[j];
          t = std::max(t, T(mods[i], lv[i]) * (1.0 + delta_of(P.e, k, peers)));
        }
      }
      if (t < best->t) {
        best->t = t;
        for (size_t i = 0; i < mods.size(); ++i) best->level[mods[i]] = lv[i];
      }
      return;
    }
    for (int p = 0; p < P.np; ++p) {
      if (used + P.cus[p] > P.total) continue;
      lv[k] = p;
      walk_rectified(k + 1, used + P.cus[p], lv, best);
    }
  }

  Eval solve() const {
    Eval ev;
    ev.t = kInf;
    for (int m = 0; m < kMaxModules; ++m) ev.level[m] = -1;
    int lv[kMaxModules];
    if (P.rect && mods.size() >= 2) {
      walk_rectified(0, 0, lv, &ev);
      return ev;
    }
    std::vector<double> cand;
    for (int m : mods) for (int p = 0; p < P.np; ++p) cand.push_back(T(m, p));
    std::sort(cand.begin(), cand.end());
    cand.erase(std::unique(cand.begin(), cand.end()), cand.end());
    if (cand.empty() || !feasible_separable(cand.back())) return ev;
    size_t lo = 0, hi = cand.size() - 1;       // invariant: cand[hi] feasible
    while (lo < hi) {
      const size_t mid = (lo + hi) / 2;
      if (feasible_separable(cand[mid])) hi = mid; else lo = mid + 1;
    }
    ev.t = cand[hi];
    if (first_tuple(0, 0, ev.t, lv))
      for (size_t i = 0; i < mods.size(); ++i) ev.level[mods[i]] = lv[i];
    return ev;
  }
};

struct Planner {
  const Problem& P;
  int flags;
  std::map<uint32_t, Eval> cache;
  mosaic_planner_stats st{0, 0, 0, 0};
  Planner(const Problem& p, int f) : P(p), flags(f) {}

  Eval eval(uint32_t mask) {
    if (flags & MOSAIC_PLANNER_CACHE) {
      auto it = cache.find(mask);
      if (it != cache.end()) { ++st.cache_hits; return it->second; }
    }
    ++st.stage_evals;
    Eval ev = StageSolver(P, mask).solve();
    if (flags & MOSAIC_PLANNER_CACHE) cache[mask] = ev;
    return ev;
  }

  // ---- the stage list and its order -------------------------------------------------------
  // A plan in the making is a list of disjoint module sets (bit masks) kept in an execution
  // order.  Everything the search needs to know about the order is one word per stage:
  // after[i] = the stages that must run after stage i, i.e. the transitive closure of "a module
  // of i feeds a module of j".  Two stages may be merged exactly when neither is in the
  // other's word (otherwise a third stage, or an edge between the two, would end up both
  // before and after the merged stage).
  struct StageList {
    std::vector<uint32_t> mask;      // modules of each stage, in execution order
    std::vector<uint32_t> after;     // bit j: stage j depends, directly or not, on stage i
  };

  // direct successors of every stage, as bit masks over stage indices
  std::vector<uint32_t> successors(const std::vector<uint32_t>& mask) const {
    std::vector<int> where(P.n, -1);
    for (size_t i = 0; i < mask.size(); ++i)
      for (int m = 0; m < P.n; ++m) if (mask[i] >> m & 1) where[m] = (int)i;
    std::vector<uint32_t> succ(mask.size(), 0);
    for (auto& ed : P.edges)
      if (where[ed.first] != where[ed.second]) succ[where[ed.first]] |= 1u << where[ed.second];
    return succ;
  }

  // Puts the stages into the order Kahn's algorithm gives when, among the stages whose
  // predecessors are all placed, the one holding the smallest module index goes first, and
  // fills `after`.  False when the stage graph has a cycle.
  bool order(StageList* L) const {
    const size_t S = L->mask.size();
    const std::vector<uint32_t> succ = successors(L->mask);
    std::vector<int> waiting(S, 0);
    for (size_t a = 0; a < S; ++a)
      for (size_t b = 0; b < S; ++b) if (succ[a] >> b & 1) ++waiting[b];
    std::vector<int> perm;                       // perm[k] = old index of the stage placed k-th
    uint32_t placed = 0;
    while (perm.size() < S) {
      int pick = -1;
      for (size_t i = 0; i < S; ++i) {
        if ((placed >> i & 1) || waiting[i] != 0) continue;
        if (pick < 0 || __builtin_ctz(L->mask[i]) < __builtin_ctz(L->mask[pick])) pick = (int)i;
      }
      if (pick < 0) return false;
      placed |= 1u << pick;
      perm.push_back(pick);
      for (size_t b = 0; b < S; ++b) if (succ[pick] >> b & 1) --waiting[b];
    }
    std::vector<int> new_index(S);
    for (size_t k = 0; k < S; ++k) new_index[perm[k]] = (int)k;
    StageList out;
    out.mask.resize(S); out.after.assign(S, 0);
    for (size_t k = 0; k < S; ++k) out.mask[k] = L->mask[perm[k]];
    // closure from the back of the order: a stage's word is its successors plus theirs
    for (int k = (int)S - 1; k >= 0; --k) {
      uint32_t w = 0;
      for (size_t b = 0; b < S; ++b)
        if (succ[perm[k]] >> b & 1) w |= (1u << new_index[b]) | out.after[new_index[b]];
      out.after[k] = w;
    }
    *L = out;
    return true;
  }

  // Early pruning: the merge can only beat `bound` = T_x + T_y - (best saving so far) if every
  // module of the merged stage has at least one level whose own time is below that bound
  // (a delay term can only be trusted not to shorten a time when its coefficients are >= 0).
  bool hopeless(uint32_t merged, double bound) const {
    if (P.rect && (P.e[0] < 0 || P.e[1] < 0 || P.e[2] < 0)) return false;
    for (int m = 0; m < P.n; ++m) {
      if (!(merged >> m & 1)) continue;
      bool any = false;
      for (int p = 0; p < P.np && !any; ++p) any = P.cus[p] <= P.total && P.t[(size_t)m * P.np + p] < bound;
      if (!any) return true;
    }
    return false;
  }

  // One merge proposal: the two stages (positions in the list), the merged set and what the
  // merge saves.  best_merge() looks at every pair the order allows, in list order, and keeps
  // the first one with the largest saving above zero.
  struct Merge { int x = -1, y = -1; uint32_t mask = 0; double saving = 0.0; Eval ev{}; };

  Merge best_merge(const StageList& L, const std::map<uint32_t, Eval>& known) {
    Merge best;
    const int S = (int)L.mask.size();
    for (int x = 0; x < S; ++x) {
      // stages that neither follow x nor are followed by it; only those behind x in the list
      uint32_t free_of_x = 0;
      for (int y = x + 1; y < S; ++y)
        if (!(L.after[x] >> y & 1) && !(L.after[y] >> x & 1)) free_of_x |= 1u << y;
      const double tx = known.at(L.mask[x]).t;
      for (int y = x + 1; y < S; ++y) {
        if (!(free_of_x >> y & 1)) continue;
        const uint32_t u = L.mask[x] | L.mask[y];
        const double apart = tx + known.at(L.mask[y]).t;
        if ((flags & MOSAIC_PLANNER_EARLY_PRUNE) && hopeless(u, apart - best.saving)) { ++st.pruned; continue; }
        const Eval ev = eval(u);
        if (apart - ev.t > best.saving) { best.x = x; best.y = y; best.mask = u; best.saving = apart - ev.t; best.ev = ev; }
      }
    }
    return best;
  }

  // Alg. 1: every module its own stage; merge while some merge saves time.
  bool run(std::vector<uint32_t>* stages_out, std::vector<Eval>* evals_out) {
    StageList L;
    for (int m = 0; m < P.n; ++m) L.mask.push_back(1u << m);
    if (!order(&L)) return false;
    std::map<uint32_t, Eval> known;            // evaluations of the stages in the list
    for (uint32_t s : L.mask) known[s] = eval(s);
    while (L.mask.size() > 1) {
      ++st.rounds;
      const Merge mg = best_merge(L, known);
      if (mg.x < 0) break;
      known[mg.mask] = mg.ev;
      L.mask[mg.x] = mg.mask;                  // the merged stage takes the place of the first
      L.mask.erase(L.mask.begin() + mg.y);
      if (!order(&L)) return false;
    }
    *stages_out = L.mask;
    evals_out->clear();
    for (uint32_t s : L.mask) evals_out->push_back(known[s]);
    return true;
  }
};

mosaic_status load_problem(const mosaic_planner_problem* pp, Problem* P) {
  if (!pp || !pp->cu_points || !pp->times) MOSAIC_FAIL(MOSAIC_EINVAL, "null planner problem");
  if (pp->n_modules < 1 || pp->n_modules > kMaxModules) MOSAIC_FAIL(MOSAIC_EINVAL, "planner handles 1..%d modules, got %d", kMaxModules, pp->n_modules);
  if (pp->n_points < 1 || pp->n_points > kMaxPoints) MOSAIC_FAIL(MOSAIC_EINVAL, "planner handles 1..%d quota levels, got %d", kMaxPoints, pp->n_points);
  if (pp->cu_total < 1) MOSAIC_FAIL(MOSAIC_EQUOTA, "cu_total %d", pp->cu_total);
  if (pp->delay_form != MOSAIC_DELAY_ABSOLUTE && pp->delay_form != MOSAIC_DELAY_PEER_RELATIVE) MOSAIC_FAIL(MOSAIC_EINVAL, "bad delay form %d", pp->delay_form);
  if (pp->n_edges < 0 || (pp->n_edges > 0 && !pp->edges)) MOSAIC_FAIL(MOSAIC_EINVAL, "bad edge list");
  if ((pp->bw == nullptr) != (pp->e == nullptr)) MOSAIC_FAIL(MOSAIC_EINVAL, "bandwidth table and coefficients are given together or not at all");
  P->n = pp->n_modules; P->np = pp->n_points; P->total = pp->cu_total; P->form = pp->delay_form;
  P->cus.assign(pp->cu_points, pp->cu_points + pp->n_points);
  for (int c : P->cus) if (c < 1) MOSAIC_FAIL(MOSAIC_EQUOTA, "quota level %d", c);
  const size_t cells = (size_t)P->n * P->np;
  P->t.assign(pp->times, pp->times + cells);
  for (double v : P->t) if (!(v >= 0.0)) MOSAIC_FAIL(MOSAIC_EINVAL, "times must be non-negative numbers");
  P->rect = pp->bw != nullptr;
  if (P->rect) {
    P->bw.assign(pp->bw, pp->bw + cells);
    for (double v : P->bw) if (!(v >= 0.0 && v <= 1.0)) MOSAIC_FAIL(MOSAIC_EINVAL, "bandwidth utilisation must lie in [0,1]");
    memcpy(P->e, pp->e, sizeof(P->e));
  } else {
    P->e[0] = P->e[1] = P->e[2] = 0.0;
  }
  for (int i = 0; i < pp->n_edges; ++i) {
    const int a = pp->edges[2 * i], b = pp->edges[2 * i + 1];
    if (a < 0 || b < 0 || a >= P->n || b >= P->n || a == b) MOSAIC_FAIL(MOSAIC_EINVAL, "edge %d: (%d,%d)", i, a, b);
    P->edges.emplace_back(a, b);
  }
  return MOSAIC_OK;
}

}  // namespace

extern "C" double mosaic_interference_delta(const double* e, int32_t k, const double* bw) {
  if (!e || k < 0 || (k > 0 && !bw)) return nan("");
  return delta_of(e, k, bw);
}

extern "C" mosaic_status mosaic_interference_fit(int32_t n_obs, const int32_t* group_size, const double* bw,
                                                 const double* delta_ms, int32_t model, double* e_out, double* r2_out) {
  if (n_obs < 1 || !group_size || !bw || !delta_ms || !e_out) MOSAIC_FAIL(MOSAIC_EINVAL, "null or empty observation list");
  if (model != MOSAIC_INTERFERENCE_ADDITIVE && model != MOSAIC_INTERFERENCE_COMPOSITE) MOSAIC_FAIL(MOSAIC_EINVAL, "bad model %d", model);
  const int nc = model == MOSAIC_INTERFERENCE_COMPOSITE ? 3 : 2;
  std::vector<double> X((size_t)n_obs * 3);
  size_t at = 0;
  for (int i = 0; i < n_obs; ++i) {
    if (group_size[i] < 1) MOSAIC_FAIL(MOSAIC_EINVAL, "observation %d has no modules", i);
    double s = 0.0, p = 1.0;
    for (int j = 0; j < group_size[i]; ++j) { s += bw[at + j]; p *= bw[at + j]; }
    at += group_size[i];
    X[3 * (size_t)i] = 1.0; X[3 * (size_t)i + 1] = s; X[3 * (size_t)i + 2] = p;
  }
  // Normal equations on centred, scaled columns would be better conditioned; three
  // columns in double are well within reach of the plain form.
  double A[3][3] = {{0}}, b[3] = {0}, x[3] = {0, 0, 0};
  for (int i = 0; i < n_obs; ++i)
    for (int r = 0; r < nc; ++r) {
      b[r] += X[3 * (size_t)i + r] * delta_ms[i];
      for (int c = 0; c < nc; ++c) A[r][c] += X[3 * (size_t)i + r] * X[3 * (size_t)i + c];
    }
  if (!solve_small(nc, A, b, x)) MOSAIC_FAIL(MOSAIC_EINVAL, "observations do not determine the coefficients");
  e_out[0] = x[0]; e_out[1] = x[1]; e_out[2] = nc == 3 ? x[2] : 0.0;
  if (r2_out) {
    double mean = 0.0;
    for (int i = 0; i < n_obs; ++i) mean += delta_ms[i];
    mean /= n_obs;
    double ss_res = 0.0, ss_tot = 0.0;
    for (int i = 0; i < n_obs; ++i) {
      const double pred = e_out[0] + e_out[1] * X[3 * (size_t)i + 1] + e_out[2] * X[3 * (size_t)i + 2];
      ss_res += (delta_ms[i] - pred) * (delta_ms[i] - pred);
      ss_tot += (delta_ms[i] - mean) * (delta_ms[i] - mean);
    }
    *r2_out = ss_tot > 0 ? 1.0 - ss_res / ss_tot : (ss_res == 0 ? 1.0 : -kInf);
  }
  return MOSAIC_OK;
}

extern "C" mosaic_status mosaic_stage_eval(const mosaic_planner_problem* pp, uint32_t module_mask,
                                           int32_t* quota_out, double* t_out) {
  Problem P;
  MOSAIC_TRY(load_problem(pp, &P));
  if (module_mask == 0 || (P.n < 32 && (module_mask >> P.n) != 0)) MOSAIC_FAIL(MOSAIC_EINVAL, "module mask 0x%x", module_mask);
  if (!quota_out || !t_out) MOSAIC_FAIL(MOSAIC_EINVAL, "null output");
  const Eval ev = StageSolver(P, module_mask).solve();
  *t_out = ev.t;
  for (int m = 0; m < P.n; ++m) quota_out[m] = ev.level[m] >= 0 ? P.cus[ev.level[m]] : 0;
  return MOSAIC_OK;
}

extern "C" mosaic_status mosaic_planner_solve(const mosaic_planner_problem* pp, int32_t flags, int32_t* stage_of,
                                              int32_t* quota_of, int32_t* n_stages, double* t_iter,
                                              mosaic_planner_stats* stats) {
  Problem P;
  MOSAIC_TRY(load_problem(pp, &P));
  if (!stage_of || !quota_of || !t_iter) MOSAIC_FAIL(MOSAIC_EINVAL, "null output");
  Planner pl(P, flags);
  std::vector<uint32_t> stages;
  std::vector<Eval> evals;
  if (!pl.run(&stages, &evals)) MOSAIC_FAIL(MOSAIC_EINVAL, "the dependency edges contain a cycle");
  double total = 0.0;
  for (size_t i = 0; i < stages.size(); ++i) {
    total += evals[i].t;                        // Eq. 1: stages follow one another in time
    for (int m = 0; m < P.n; ++m)
      if (stages[i] >> m & 1) {
        stage_of[m] = (int32_t)i;
        quota_of[m] = evals[i].level[m] >= 0 ? P.cus[evals[i].level[m]] : 0;
      }
  }
  *t_iter = total;
  if (n_stages) *n_stages = (int32_t)stages.size();
  if (stats) *stats = pl.st;
  return MOSAIC_OK;
}
