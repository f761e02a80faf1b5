// Host-side plan search of Strand Interleaving (paper Sec. 4.2): overlap effectiveness (Eq. 1),
// the pairing recurrence (Eq. 2), the segment-pair cost model, operator sequencing and barrier
// placement.  No device code.
#include <algorithm>
#include <cstring>
#include <limits>
#include <vector>
#include "common.h"

extern "C" double dh_oef(double t_i, double t_j, double p_ij) { return (t_i + t_j - p_ij) / std::min(t_i, t_j); }

// Two-queue fluid model.  While forward operator a and backward operator b are both running they
// advance at the profiled rates; when one finishes the next operator of its strand starts at once;
// when one strand runs dry the other proceeds undisturbed.
static double segment_cost(const dh_overlap_table& t, const int* sf, int nf, const int* sb, int nb) {
  int fi = 0, bi = 0;
  double now = 0.0;
  double left_f = nf > 0 ? t.t_fwd[sf[0]] : 0.0, left_b = nb > 0 ? t.t_bwd[sb[0]] : 0.0;
  while (fi < nf && bi < nb) {
    const double rf = t.rate_fwd[sf[fi]][sb[bi]], rb = t.rate_bwd[sf[fi]][sb[bi]];
    const double need_f = left_f / rf, need_b = left_b / rb;
    const double dt = std::min(need_f, need_b);
    now += dt;
    left_f -= rf * dt;
    left_b -= rb * dt;
    const bool f_done = need_f <= need_b, b_done = need_b <= need_f;
    if (f_done) { ++fi; left_f = fi < nf ? t.t_fwd[sf[fi]] : 0.0; }
    if (b_done) { ++bi; left_b = bi < nb ? t.t_bwd[sb[bi]] : 0.0; }
  }
  if (fi < nf) { now += left_f; for (int k = fi + 1; k < nf; k++) now += t.t_fwd[sf[k]]; }
  if (bi < nb) { now += left_b; for (int k = bi + 1; k < nb; k++) now += t.t_bwd[sb[k]]; }
  return now;
}

static int check_table_ids(const dh_overlap_table* t, const int* sf, int nf, const int* sb, int nb) {
  if (!t || nf < 0 || nb < 0 || (nf > 0 && !sf) || (nb > 0 && !sb)) return DH_ERR_INVALID_ARG;
  if (t->n_fwd < 0 || t->n_fwd > DH_MAX_OPS || t->n_bwd < 0 || t->n_bwd > DH_MAX_OPS) return DH_ERR_INVALID_ARG;
  for (int i = 0; i < nf; i++) if (sf[i] < 0 || sf[i] >= t->n_fwd) return DH_ERR_INVALID_ARG;
  for (int j = 0; j < nb; j++) if (sb[j] < 0 || sb[j] >= t->n_bwd) return DH_ERR_INVALID_ARG;
  for (int i = 0; i < nf; i++)
    for (int j = 0; j < nb; j++)
      if (!(t->rate_fwd[sf[i]][sb[j]] > 0.0) || !(t->rate_bwd[sf[i]][sb[j]] > 0.0)) return DH_ERR_INVALID_ARG;
  return DH_OK;
}

extern "C" double dh_segment_cost(const dh_overlap_table* t, const int* seg_f, int n_f, const int* seg_b, int n_b) {
  int rc = check_table_ids(t, seg_f, n_f, seg_b, n_b);
  if (rc != DH_OK) {
    dh_set_error(rc, "segment_cost: bad table, operator id or non-positive rate");
    return (double)rc;
  }
  return segment_cost(*t, seg_f, n_f, seg_b, n_b);
}

// Eq. 2 over prefixes of the two segment lists; ties prefer pairing, then forward-alone.
extern "C" int dh_pair_dp(const double* p_f, int n_f, const double* p_b, int n_b, const double* p_fb, double* t_opt,
                          int* steps, int* n_steps) {
  if (n_f < 0 || n_b < 0 || !t_opt || (n_f > 0 && !p_f) || (n_b > 0 && !p_b) || (n_f > 0 && n_b > 0 && !p_fb))
    DH_FAIL(DH_ERR_INVALID_ARG, "pair_dp: bad arguments");
  const int W = n_b + 1;
  std::vector<double> T((size_t)(n_f + 1) * W, std::numeric_limits<double>::infinity());
  std::vector<signed char> how((size_t)(n_f + 1) * W, -1);  // 0 pair, 1 forward alone, 2 backward alone
  T[0] = 0.0;
  for (int i = 0; i <= n_f; i++)
    for (int j = 0; j <= n_b; j++) {
      if (i == 0 && j == 0) continue;
      double best = std::numeric_limits<double>::infinity();
      signed char hb = -1;
      if (i > 0 && j > 0) { double c = T[(i - 1) * W + j - 1] + p_fb[(size_t)(i - 1) * n_b + j - 1]; if (c < best) { best = c; hb = 0; } }
      if (i > 0) { double c = T[(i - 1) * W + j] + p_f[i - 1]; if (c < best) { best = c; hb = 1; } }
      if (j > 0) { double c = T[i * W + j - 1] + p_b[j - 1]; if (c < best) { best = c; hb = 2; } }
      T[i * W + j] = best;
      how[i * W + j] = hb;
    }
  *t_opt = T[(size_t)n_f * W + n_b];
  if (steps && n_steps) {
    std::vector<std::pair<int, int>> rev;
    int i = n_f, j = n_b;
    while (i > 0 || j > 0) {
      signed char h = how[i * W + j];
      if (h == 0) { rev.push_back({i - 1, j - 1}); --i; --j; }
      else if (h == 1) { rev.push_back({i - 1, -1}); --i; }
      else { rev.push_back({-1, j - 1}); --j; }
    }
    *n_steps = (int)rev.size();
    for (size_t k = 0; k < rev.size(); k++) {
      steps[2 * k] = rev[rev.size() - 1 - k].first;
      steps[2 * k + 1] = rev[rev.size() - 1 - k].second;
    }
  }
  return DH_OK;
}

static int check_graph(const dh_op_graph* g) {
  if (!g || g->n_ops < 0 || g->n_ops > DH_MAX_OPS || g->n_deps < 0 || g->n_deps > DH_MAX_DEPS) return DH_ERR_INVALID_ARG;
  for (int e = 0; e < g->n_deps; e++)
    if (g->dep_src[e] < 0 || g->dep_src[e] >= g->n_ops || g->dep_dst[e] < 0 || g->dep_dst[e] >= g->n_ops) return DH_ERR_INVALID_ARG;
  return DH_OK;
}

// Depth-first enumeration of topological orders, smallest operator id first, capped.
static void enum_orders(const dh_op_graph& g, int cap, std::vector<std::vector<int>>& out) {
  const int n = g.n_ops;
  std::vector<int> indeg(n, 0), cur;
  std::vector<char> used(n, 0);
  for (int e = 0; e < g.n_deps; e++) indeg[g.dep_dst[e]]++;
  struct Rec {
    const dh_op_graph& g; int cap; std::vector<std::vector<int>>& out;
    std::vector<int>& indeg; std::vector<char>& used; std::vector<int>& cur;
    void go() {
      if ((int)out.size() >= cap) return;
      if ((int)cur.size() == g.n_ops) { out.push_back(cur); return; }
      for (int v = 0; v < g.n_ops; v++) {
        if (used[v] || indeg[v] != 0) continue;
        used[v] = 1; cur.push_back(v);
        for (int e = 0; e < g.n_deps; e++) if (g.dep_src[e] == v) indeg[g.dep_dst[e]]--;
        go();
        for (int e = 0; e < g.n_deps; e++) if (g.dep_src[e] == v) indeg[g.dep_dst[e]]++;
        cur.pop_back(); used[v] = 0;
        if ((int)out.size() >= cap) return;
      }
    }
  } rec{g, cap, out, indeg, used, cur};
  rec.go();
}

// Barrier placement for fixed sequences: T(i,j) = min over (i',j') != (i,j), i'<=i, j'<=j of
// T(i',j') + cost(seq_f[i':i], seq_b[j':j]) + barrier.
static double place_barriers(const dh_overlap_table& t, const std::vector<int>& sf, const std::vector<int>& sb,
                             double barrier, std::vector<dh_seg_pair>* pairs) {
  const int nf = (int)sf.size(), nb = (int)sb.size(), W = nb + 1;
  std::vector<double> T((size_t)(nf + 1) * W, std::numeric_limits<double>::infinity());
  std::vector<int> from((size_t)(nf + 1) * W, -1);
  T[0] = 0.0;
  for (int i = 0; i <= nf; i++)
    for (int j = 0; j <= nb; j++) {
      if (i == 0 && j == 0) continue;
      double best = std::numeric_limits<double>::infinity();
      int bf = -1;
      for (int ip = 0; ip <= i; ip++)
        for (int jp = 0; jp <= j; jp++) {
          if (ip == i && jp == j) continue;
          double c = T[ip * W + jp] + segment_cost(t, sf.data() + ip, i - ip, sb.data() + jp, j - jp) + barrier;
          if (c < best) { best = c; bf = ip * W + jp; }
        }
      T[i * W + j] = best;
      from[i * W + j] = bf;
    }
  if (pairs) {
    pairs->clear();
    int i = nf, j = nb;
    while (i > 0 || j > 0) {
      int f = from[i * W + j], ip = f / W, jp = f % W;
      pairs->push_back({ip, i, jp, j});
      i = ip; j = jp;
    }
    std::reverse(pairs->begin(), pairs->end());
  }
  return T[(size_t)nf * W + nb];
}

extern "C" int dh_plan_validate(const dh_op_graph* fwd, const dh_op_graph* bwd, const dh_plan* plan) {
  if (check_graph(fwd) != DH_OK || check_graph(bwd) != DH_OK || !plan) DH_FAIL(DH_ERR_INVALID_ARG, "plan_validate: bad arguments");
  if (plan->n_fwd != fwd->n_ops || plan->n_bwd != bwd->n_ops) DH_FAIL(DH_ERR_PLAN_INVALID, "plan: operator counts %d/%d do not match the graphs %d/%d", plan->n_fwd, plan->n_bwd, fwd->n_ops, bwd->n_ops);
  auto check_order = [](const dh_op_graph* g, const int* order, const char* side) -> int {
    int pos[DH_MAX_OPS];
    for (int i = 0; i < g->n_ops; i++) pos[i] = -1;
    for (int i = 0; i < g->n_ops; i++) {
      int v = order[i];
      if (v < 0 || v >= g->n_ops || pos[v] >= 0) return dh_set_error(DH_ERR_PLAN_INVALID, "plan: %s order is not a permutation (entry %d)", side, i);
      pos[v] = i;
    }
    for (int e = 0; e < g->n_deps; e++)
      if (pos[g->dep_src[e]] > pos[g->dep_dst[e]])
        return dh_set_error(DH_ERR_PLAN_INVALID, "plan: %s order runs operator %d before its input %d", side, g->dep_dst[e], g->dep_src[e]);
    return DH_OK;
  };
  int rc = check_order(fwd, plan->fwd_order, "forward");
  if (rc) return rc;
  rc = check_order(bwd, plan->bwd_order, "backward");
  if (rc) return rc;
  if (plan->n_pairs < 0 || plan->n_pairs > 2 * DH_MAX_OPS) DH_FAIL(DH_ERR_PLAN_INVALID, "plan: %d segment pairs", plan->n_pairs);
  int fi = 0, bj = 0;
  for (int k = 0; k < plan->n_pairs; k++) {
    const dh_seg_pair& p = plan->pairs[k];
    if (p.f_begin != fi || p.b_begin != bj || p.f_end < p.f_begin || p.b_end < p.b_begin || p.f_end > plan->n_fwd || p.b_end > plan->n_bwd)
      DH_FAIL(DH_ERR_PLAN_INVALID, "plan: segment pair %d does not continue the tiling", k);
    fi = p.f_end; bj = p.b_end;
  }
  if (fi != plan->n_fwd || bj != plan->n_bwd) DH_FAIL(DH_ERR_PLAN_INVALID, "plan: segment pairs cover %d/%d of %d/%d operators", fi, bj, plan->n_fwd, plan->n_bwd);
  for (int op = 0; op < DH_MAX_OPS; op++)
    if (plan->bwd_side[op] && (op >= bwd->n_ops || !bwd->side_ok[op]))
      DH_FAIL(DH_ERR_PLAN_INVALID, "plan: backward operator %d may not run beside its strand", op);
  return DH_OK;
}

extern "C" int dh_plan_search(const dh_op_graph* fwd, const dh_op_graph* bwd, const dh_overlap_table* table,
                              double barrier_cost, int max_orders, dh_plan* out, double* makespan) {
  if (check_graph(fwd) != DH_OK || check_graph(bwd) != DH_OK || !table || !out || !makespan || barrier_cost < 0)
    DH_FAIL(DH_ERR_INVALID_ARG, "plan_search: bad arguments");
  if (table->n_fwd < fwd->n_ops || table->n_bwd < bwd->n_ops) DH_FAIL(DH_ERR_INVALID_ARG, "plan_search: table smaller than the graphs");
  for (int i = 0; i < fwd->n_ops; i++)
    for (int j = 0; j < bwd->n_ops; j++)
      if (!(table->rate_fwd[i][j] > 0.0) || !(table->rate_bwd[i][j] > 0.0)) DH_FAIL(DH_ERR_INVALID_ARG, "plan_search: non-positive rate at (%d,%d)", i, j);
  if (max_orders <= 0) max_orders = 512;
  std::vector<std::vector<int>> of, ob;
  enum_orders(*fwd, max_orders, of);
  enum_orders(*bwd, max_orders, ob);
  if (of.empty() || ob.empty()) DH_FAIL(DH_ERR_PLAN_INVALID, "plan_search: an operator graph has a cycle");
  double best = std::numeric_limits<double>::infinity();
  size_t bi = 0, bj = 0;
  for (size_t a = 0; a < of.size(); a++)
    for (size_t b = 0; b < ob.size(); b++) {
      double m = place_barriers(*table, of[a], ob[b], barrier_cost, nullptr);
      if (m < best) { best = m; bi = a; bj = b; }
    }
  std::vector<dh_seg_pair> pairs;
  place_barriers(*table, of[bi], ob[bj], barrier_cost, &pairs);
  out->n_fwd = fwd->n_ops;
  out->n_bwd = bwd->n_ops;
  for (int i = 0; i < fwd->n_ops; i++) out->fwd_order[i] = of[bi][i];
  for (int j = 0; j < bwd->n_ops; j++) out->bwd_order[j] = ob[bj][j];
  out->n_pairs = (int)pairs.size();
  for (size_t k = 0; k < pairs.size(); k++) out->pairs[k] = pairs[k];
  *makespan = best;
  return DH_OK;
}

// The comparison schedule of Sec. 6.1 ("Wavelet+"): the two strands' operators are interleaved one by one in
// their default orders, with a barrier after every pair, and no operator is moved.
extern "C" int dh_plan_round_robin(const dh_op_graph* fwd, const dh_op_graph* bwd, dh_plan* out) {
  if (!fwd || !bwd || !out) DH_FAIL(DH_ERR_INVALID_ARG, "plan_round_robin: null pointer");
  if (fwd->n_ops < 0 || fwd->n_ops > DH_MAX_OPS || bwd->n_ops < 0 || bwd->n_ops > DH_MAX_OPS)
    DH_FAIL(DH_ERR_INVALID_ARG, "plan_round_robin: operator count out of range");
  std::vector<std::vector<int>> of, ob;
  enum_orders(*fwd, 1, of);
  enum_orders(*bwd, 1, ob);
  if (of.empty() || ob.empty()) DH_FAIL(DH_ERR_PLAN_INVALID, "plan_round_robin: an operator graph has a cycle");
  memset(out, 0, sizeof(*out));
  out->n_fwd = fwd->n_ops;
  out->n_bwd = bwd->n_ops;
  for (int i = 0; i < fwd->n_ops; i++) out->fwd_order[i] = of[0][i];
  for (int j = 0; j < bwd->n_ops; j++) out->bwd_order[j] = ob[0][j];
  const int n = std::max(fwd->n_ops, bwd->n_ops);
  out->n_pairs = n;
  for (int k = 0; k < n; k++)
    out->pairs[k] = {std::min(k, fwd->n_ops), std::min(k + 1, fwd->n_ops), std::min(k, bwd->n_ops), std::min(k + 1, bwd->n_ops)};
  return DH_OK;
}
