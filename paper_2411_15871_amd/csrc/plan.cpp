// Host-side plan search of Strand Interleaving (paper Sec. 4.2): overlap effectiveness (Eq. 1),
// the pairing recurrence (Eq. 2), the segment-pair cost model, operator sequencing and barrier
// placement.  No device code.
#include <algorithm>
#include <cstring>
#include <limits>
#include <thread>
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

static void search_orders(const dh_op_graph& g, int cap, std::vector<std::vector<int>>& out, long long* total);

extern "C" int dh_plan_search(const dh_op_graph* fwd, const dh_op_graph* bwd, const dh_overlap_table* table,
                              double barrier_cost, int max_orders, dh_plan* out, double* makespan) {
  if (check_graph(fwd) != DH_OK || check_graph(bwd) != DH_OK || !table || !out || !makespan || barrier_cost < 0)
    DH_FAIL(DH_ERR_INVALID_ARG, "plan_search: bad arguments");
  if (table->n_fwd < fwd->n_ops || table->n_bwd < bwd->n_ops) DH_FAIL(DH_ERR_INVALID_ARG, "plan_search: table smaller than the graphs");
  for (int i = 0; i < fwd->n_ops; i++)
    for (int j = 0; j < bwd->n_ops; j++)
      if (!(table->rate_fwd[i][j] > 0.0) || !(table->rate_bwd[i][j] > 0.0)) DH_FAIL(DH_ERR_INVALID_ARG, "plan_search: non-positive rate at (%d,%d)", i, j);
  if (max_orders <= 0) max_orders = 20000;  // every order of the layers' graphs (5760 for the Llama backward graph); dh_plan_count_orders tells
  std::vector<std::vector<int>> of, ob;
  long long tot_f = 0, tot_b = 0;
  search_orders(*fwd, max_orders, of, &tot_f);
  search_orders(*bwd, max_orders, ob, &tot_b);
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

// ------------------------------------------------------------------------------------ lane model
// Cost of a segment pair as dh_si_step runs it.  The two-queue model above knows two participants; the executor has
// up to five streams ("lanes"): the two strands, a communication stream (shared, or one per strand) and the cross-node
// stream.  A stand-in issued on another lane than its strand's starts when everything its strand has issued so far
// is done, and the strand waits for it only before an operator that consumes its result (operator graph) -- so weight
// gradients overlap their own strand's collective (Sec. 4.2: the movable, "self-overlapping" operators), and an
// operator flagged bwd_side runs on alpha's lane once beta's operators before it are done.  The model replays exactly
// that issue logic as a dependency graph over lanes (a lane runs its operators in issue order) and integrates it as a
// fluid: an active operator advances at the product of the pairwise rates of the table against every other active
// operator.  Pairs of one direction are not in the table (the profiler co-runs forward with backward operators); they
// are looked up through the operator of the other direction that runs the same kernel on the same data size
// (dh_op_graph.like_other), and count as undisturbed (rate 1) when there is none.
namespace {
enum { LANE_A = 0, LANE_B = 1, LANE_COMM = 2, LANE_COMM_B = 3, LANE_CROSS = 4, N_LANES = 5 };
struct Node {
  int dir, op, lane;
  double work;
  int ndep;
  int dep[4 + DH_MAX_OPS];  // nodes that must have finished (besides the lane's previous node)
};
struct LaneSim {
  const dh_op_graph& gf;
  const dh_op_graph& gb;
  const dh_overlap_table& t;
  dh_lanes lanes;
  std::vector<Node> nodes;
  std::vector<int> lane_nodes[N_LANES];
  LaneSim(const dh_op_graph& f, const dh_op_graph& b, const dh_overlap_table& tab, const dh_lanes& l) : gf(f), gb(b), t(tab), lanes(l) {}

  int comm_lane(int dir, int kind) const {
    if (kind == 2 && lanes.cross) return LANE_CROSS;
    if (dir == 0) return lanes.comm_alpha ? LANE_COMM : LANE_A;
    return lanes.comm_beta == 0 ? LANE_B : lanes.comm_beta == 1 ? LANE_COMM : LANE_COMM_B;
  }
  // rate of x while y is active
  double pair_rate(const Node& x, const Node& y) const {
    int xd = x.dir, xo = x.op, yd = y.dir, yo = y.op;
    if (xd == yd) {  // same direction: stand in the like operator of the other direction for one of them
      const dh_op_graph& g = xd == 0 ? gf : gb;
      if (g.like_other[yo] > 0) { yd = 1 - yd; yo = g.like_other[yo] - 1; }
      else if (g.like_other[xo] > 0) { xd = 1 - xd; xo = g.like_other[xo] - 1; }
      else return 1.0;
    }
    return xd == 0 ? t.rate_fwd[xo][yo] : t.rate_bwd[yo][xo];
  }
  // Builds the nodes of one segment pair the way dh_si_step issues it (alternating forward and backward operators).
  void build(const int* fo, int nf, const int* bo, int nb, const int* side) {
    nodes.clear();
    for (auto& v : lane_nodes) v.clear();
    int pend_f[DH_MAX_OPS], pend_b[DH_MAX_OPS];  // node of a stand-in its strand has not waited for yet, or -1
    for (int i = 0; i < DH_MAX_OPS; i++) pend_f[i] = pend_b[i] = -1;
    std::vector<int> carry[N_LANES];  // extra dependencies of the next node issued on a lane (stream waits)
    auto last_of = [&](int lane) { return lane_nodes[lane].empty() ? -1 : lane_nodes[lane].back(); };
    auto add = [&](int dir, int op, int lane, int extra_dep) {
      Node n;
      n.dir = dir; n.op = op; n.lane = lane; n.ndep = 0;
      n.work = dir == 0 ? t.t_fwd[op] : t.t_bwd[op];
      for (int d : carry[lane]) n.dep[n.ndep++] = d;
      carry[lane].clear();
      if (extra_dep >= 0) n.dep[n.ndep++] = extra_dep;
      nodes.push_back(n);
      lane_nodes[lane].push_back((int)nodes.size() - 1);
      return (int)nodes.size() - 1;
    };
    auto wait_inputs = [&](const dh_op_graph& g, int* pend, int op, int lane) {
      for (int e = 0; e < g.n_deps; e++)
        if (g.dep_dst[e] == op && pend[g.dep_src[e]] >= 0) { carry[lane].push_back(pend[g.dep_src[e]]); pend[g.dep_src[e]] = -1; }
    };
    int fi = 0, bj = 0;
    while (fi < nf || bj < nb) {
      if (fi < nf) {
        const int op = fo[fi++];
        wait_inputs(gf, pend_f, op, LANE_A);
        const int lane = gf.is_comm[op] ? comm_lane(0, gf.is_comm[op]) : LANE_A;
        if (lane != LANE_A) pend_f[op] = add(0, op, lane, last_of(LANE_A));
        else add(0, op, LANE_A, -1);
      }
      if (bj < nb) {
        const int op = bo[bj++];
        wait_inputs(gb, pend_b, op, LANE_B);
        if (side && side[op]) {
          // beta's lane has taken up its waits (they order the event the side operator starts behind)
          std::vector<int> deps = carry[LANE_B];
          const int n = add(1, op, LANE_A, last_of(LANE_B));
          for (int d : deps) nodes[n].dep[nodes[n].ndep++] = d;
          continue;
        }
        const int lane = gb.is_comm[op] ? comm_lane(1, gb.is_comm[op]) : LANE_B;
        if (lane != LANE_B) pend_b[op] = add(1, op, lane, last_of(LANE_B));
        else add(1, op, LANE_B, -1);
      }
    }
  }
  // Fluid integration; returns the time at which the last node finishes.
  double run() {
    const int n = (int)nodes.size();
    std::vector<double> left(n);
    std::vector<char> done(n, 0);
    for (int i = 0; i < n; i++) left[i] = nodes[i].work;
    size_t head[N_LANES] = {0, 0, 0, 0, 0};
    double now = 0.0;
    int remaining = n;
    while (remaining > 0) {
      int act[N_LANES], na = 0;
      for (int l = 0; l < N_LANES; l++) {
        while (head[l] < lane_nodes[l].size() && done[lane_nodes[l][head[l]]]) head[l]++;
        if (head[l] >= lane_nodes[l].size()) continue;
        const int v = lane_nodes[l][head[l]];
        bool ready = true;
        for (int d = 0; d < nodes[v].ndep && ready; d++) ready = done[nodes[v].dep[d]];
        if (ready) act[na++] = v;
      }
      if (na == 0) return -1.0;  // cannot happen for a validated plan
      double rate[N_LANES], dt = std::numeric_limits<double>::infinity();
      for (int a = 0; a < na; a++) {
        double r = 1.0;
        for (int b = 0; b < na; b++)
          if (b != a) r *= pair_rate(nodes[act[a]], nodes[act[b]]);
        rate[a] = r;
        dt = std::min(dt, left[act[a]] / r);
      }
      now += dt;
      for (int a = 0; a < na; a++) {
        left[act[a]] -= rate[a] * dt;
        if (left[act[a]] <= 1e-15 * (nodes[act[a]].work + 1e-300) || left[act[a]] / rate[a] <= dt * 1e-12) { done[act[a]] = 1; remaining--; }
      }
    }
    return now;
  }
  double segment(const int* fo, int nf, const int* bo, int nb, const int* side) {
    build(fo, nf, bo, nb, side);
    return run();
  }
};

int check_lanes(const dh_lanes* l) {
  if (!l || l->comm_alpha < 0 || l->comm_alpha > 1 || l->comm_beta < 0 || l->comm_beta > 2 || l->cross < 0 || l->cross > 1) return DH_ERR_INVALID_ARG;
  return DH_OK;
}
int check_table_for(const dh_op_graph* fwd, const dh_op_graph* bwd, const dh_overlap_table* table) {
  if (!table || table->n_fwd < fwd->n_ops || table->n_bwd < bwd->n_ops) return DH_ERR_INVALID_ARG;
  for (int i = 0; i < fwd->n_ops; i++)
    for (int j = 0; j < bwd->n_ops; j++)
      if (!(table->rate_fwd[i][j] > 0.0) || !(table->rate_bwd[i][j] > 0.0)) return DH_ERR_INVALID_ARG;
  for (int i = 0; i < fwd->n_ops; i++) if (fwd->like_other[i] < 0 || fwd->like_other[i] > bwd->n_ops) return DH_ERR_INVALID_ARG;
  for (int j = 0; j < bwd->n_ops; j++) if (bwd->like_other[j] < 0 || bwd->like_other[j] > fwd->n_ops) return DH_ERR_INVALID_ARG;
  return DH_OK;
}

// Barrier placement with the lane model as P: the same recurrence as place_barriers.
double place_barriers_lanes(LaneSim& sim, const std::vector<int>& sf, const std::vector<int>& sb, const int* side, double barrier,
                            std::vector<dh_seg_pair>* pairs) {
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
          if (T[ip * W + jp] + barrier >= best) continue;  // a segment pair never costs less than nothing
          const double c = T[ip * W + jp] + sim.segment(sf.data() + ip, i - ip, sb.data() + jp, j - jp, side) + barrier;
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
}  // namespace

extern "C" double dh_plan_cost(const dh_op_graph* fwd, const dh_op_graph* bwd, const dh_overlap_table* table, const dh_plan* plan,
                               const dh_lanes* lanes, double barrier_cost) {
  int rc = DH_OK;
  if (check_graph(fwd) != DH_OK || check_graph(bwd) != DH_OK || check_lanes(lanes) != DH_OK || !plan || barrier_cost < 0) rc = DH_ERR_INVALID_ARG;
  if (rc == DH_OK) rc = check_table_for(fwd, bwd, table);
  if (rc != DH_OK) { dh_set_error(rc, "plan_cost: bad graph, table, lanes or plan"); return (double)rc; }
  if ((rc = dh_plan_validate(fwd, bwd, plan)) != DH_OK) return (double)rc;
  LaneSim sim(*fwd, *bwd, *table, *lanes);
  double total = 0.0;
  for (int k = 0; k < plan->n_pairs; k++) {
    const dh_seg_pair& p = plan->pairs[k];
    total += sim.segment(plan->fwd_order + p.f_begin, p.f_end - p.f_begin, plan->bwd_order + p.b_begin, p.b_end - p.b_begin, plan->bwd_side);
    total += barrier_cost;
  }
  return total;
}

extern "C" long long dh_plan_count_orders(const dh_op_graph* g, long long cap) {
  if (check_graph(g) != DH_OK || cap <= 0) { dh_set_error(DH_ERR_INVALID_ARG, "plan_count_orders: bad arguments"); return DH_ERR_INVALID_ARG; }
  const int n = g->n_ops;
  std::vector<int> indeg(n, 0);
  std::vector<char> used(n, 0);
  for (int e = 0; e < g->n_deps; e++) indeg[g->dep_dst[e]]++;
  long long count = 0;
  struct Rec {
    const dh_op_graph& g; long long cap; long long& count; std::vector<int>& indeg; std::vector<char>& used; int depth;
    void go() {
      if (count >= cap) return;
      if (depth == g.n_ops) { count++; return; }
      for (int v = 0; v < g.n_ops && count < cap; v++) {
        if (used[v] || indeg[v] != 0) continue;
        used[v] = 1; depth++;
        for (int e = 0; e < g.n_deps; e++) if (g.dep_src[e] == v) indeg[g.dep_dst[e]]--;
        go();
        for (int e = 0; e < g.n_deps; e++) if (g.dep_src[e] == v) indeg[g.dep_dst[e]]++;
        depth--; used[v] = 0;
      }
    }
  } rec{*g, cap, count, indeg, used, 0};
  rec.go();
  return count;
}

// Orders of a graph for the search: all of them when there are at most `cap`; otherwise the first cap/2 of the
// depth-first enumeration plus cap/2 orders drawn by a seeded generator (uniform choice among the ready operators at
// every step), so that operators without successors are tried in every place and not only at the tail.
static void search_orders(const dh_op_graph& g, int cap, std::vector<std::vector<int>>& out, long long* total) {
  const long long count = dh_plan_count_orders(&g, (long long)cap + 1);
  *total = count;
  if (count <= cap) { enum_orders(g, cap, out); return; }
  enum_orders(g, (cap + 1) / 2, out);
  uint64_t state = 0x9E3779B97F4A7C15ull;
  auto next = [&]() { state = state * 6364136223846793005ull + 1442695040888963407ull; return (uint32_t)(state >> 33); };
  const int n = g.n_ops;
  for (int k = 0; k < cap - (cap + 1) / 2; k++) {
    std::vector<int> indeg(n, 0), order;
    std::vector<char> used(n, 0);
    for (int e = 0; e < g.n_deps; e++) indeg[g.dep_dst[e]]++;
    for (int step = 0; step < n; step++) {
      int ready[DH_MAX_OPS], nr = 0;
      for (int v = 0; v < n; v++) if (!used[v] && indeg[v] == 0) ready[nr++] = v;
      const int v = ready[next() % nr];
      used[v] = 1; order.push_back(v);
      for (int e = 0; e < g.n_deps; e++) if (g.dep_src[e] == v) indeg[g.dep_dst[e]]--;
    }
    out.push_back(order);
  }
}

extern "C" int dh_plan_search_lanes(const dh_op_graph* fwd, const dh_op_graph* bwd, const dh_overlap_table* table, const dh_lanes* lanes,
                                    double barrier_cost, int max_orders, dh_plan* out, double* makespan, dh_search_info* info) {
  if (check_graph(fwd) != DH_OK || check_graph(bwd) != DH_OK || check_lanes(lanes) != DH_OK || !out || !makespan || barrier_cost < 0)
    DH_FAIL(DH_ERR_INVALID_ARG, "plan_search_lanes: bad arguments");
  if (check_table_for(fwd, bwd, table) != DH_OK) DH_FAIL(DH_ERR_INVALID_ARG, "plan_search_lanes: table does not fit the graphs or holds a non-positive rate");
  if (max_orders <= 0) max_orders = 20000;
  std::vector<std::vector<int>> of, ob;
  long long tot_f = 0, tot_b = 0;
  search_orders(*fwd, std::max(1, std::min(max_orders, 64)), of, &tot_f);  // the forward graphs are (nearly) chains
  search_orders(*bwd, max_orders, ob, &tot_b);
  if (of.empty() || ob.empty()) DH_FAIL(DH_ERR_PLAN_INVALID, "plan_search_lanes: an operator graph has a cycle");
  // Step 1: every pair of orders as one free-running segment pair, with no operator beside its strand.
  struct Cand { double m; int a, b; };
  std::vector<Cand> cands(of.size() * ob.size());
  const int zero_side[DH_MAX_OPS] = {0};
  {
    const unsigned nt = std::max(1u, std::min(16u, std::thread::hardware_concurrency()));
    std::vector<std::thread> pool;
    for (unsigned w = 0; w < nt; w++)
      pool.emplace_back([&, w]() {
        LaneSim sim(*fwd, *bwd, *table, *lanes);
        for (size_t k = w; k < cands.size(); k += nt) {
          const int a = (int)(k / ob.size()), b = (int)(k % ob.size());
          cands[k] = {sim.segment(of[a].data(), fwd->n_ops, ob[b].data(), bwd->n_ops, zero_side) + barrier_cost, a, b};
        }
      });
    for (auto& th : pool) th.join();
  }
  std::stable_sort(cands.begin(), cands.end(), [](const Cand& x, const Cand& y) { return x.m < y.m; });
  // Step 2: barrier placement (Eq. 2 over prefixes) on the best orders and on a spread of the rest; for each, the
  // side_ok operators beside the strand or not (all subsets up to 4 such operators, else none / each alone / all).
  std::vector<size_t> refine;
  const size_t n_top = std::min<size_t>(cands.size(), 24), n_spread = std::min<size_t>(cands.size() - n_top, 8);
  for (size_t k = 0; k < n_top; k++) refine.push_back(k);
  for (size_t k = 0; k < n_spread; k++) refine.push_back(n_top + (cands.size() - n_top) * k / n_spread);
  std::vector<int> side_ops;
  for (int op = 0; op < bwd->n_ops; op++) if (bwd->side_ok[op]) side_ops.push_back(op);
  std::vector<std::vector<int>> subsets;
  if (side_ops.size() <= 4) {
    for (unsigned m = 0; m < (1u << side_ops.size()); m++) {
      std::vector<int> sset;
      for (size_t i = 0; i < side_ops.size(); i++) if (m >> i & 1) sset.push_back(side_ops[i]);
      subsets.push_back(sset);
    }
  } else {
    subsets.push_back({});
    for (int op : side_ops) subsets.push_back({op});
    subsets.push_back(side_ops);
  }
  struct Best { double m = std::numeric_limits<double>::infinity(); int a = 0, b = 0, subset = 0; bool dp = false; };
  std::vector<Best> bests(refine.size());
  {
    const unsigned nt = std::max(1u, std::min(16u, std::thread::hardware_concurrency()));
    std::vector<std::thread> pool;
    for (unsigned w = 0; w < nt; w++)
      pool.emplace_back([&, w]() {
        LaneSim sim(*fwd, *bwd, *table, *lanes);
        for (size_t r = w; r < refine.size(); r += nt) {
          const Cand& c = cands[refine[r]];
          Best& bb = bests[r];
          bb.a = c.a; bb.b = c.b;
          // first the subsets on the free-running pair, then barrier placement under the best subset
          for (size_t si = 0; si < subsets.size(); si++) {
            int side[DH_MAX_OPS] = {0};
            for (int op : subsets[si]) side[op] = 1;
            const double m = sim.segment(of[c.a].data(), fwd->n_ops, ob[c.b].data(), bwd->n_ops, side) + barrier_cost;
            if (m < bb.m) { bb.m = m; bb.subset = (int)si; bb.dp = false; }
          }
          int side[DH_MAX_OPS] = {0};
          for (int op : subsets[bb.subset]) side[op] = 1;
          const double m = place_barriers_lanes(sim, of[c.a], ob[c.b], side, barrier_cost, nullptr);
          if (m < bb.m) { bb.m = m; bb.dp = true; }
        }
      });
    for (auto& th : pool) th.join();
  }
  size_t win = 0;
  for (size_t r = 1; r < bests.size(); r++) if (bests[r].m < bests[win].m) win = r;
  const Best& bw = bests[win];
  memset(out, 0, sizeof(*out));
  out->n_fwd = fwd->n_ops;
  out->n_bwd = bwd->n_ops;
  for (int i = 0; i < fwd->n_ops; i++) out->fwd_order[i] = of[bw.a][i];
  for (int j = 0; j < bwd->n_ops; j++) out->bwd_order[j] = ob[bw.b][j];
  for (int op : subsets[bw.subset]) out->bwd_side[op] = 1;
  if (bw.dp) {
    LaneSim sim(*fwd, *bwd, *table, *lanes);
    std::vector<dh_seg_pair> pairs;
    place_barriers_lanes(sim, of[bw.a], ob[bw.b], out->bwd_side, barrier_cost, &pairs);
    out->n_pairs = (int)pairs.size();
    for (size_t k = 0; k < pairs.size(); k++) out->pairs[k] = pairs[k];
  } else {
    out->n_pairs = 1;
    out->pairs[0] = {0, fwd->n_ops, 0, bwd->n_ops};
  }
  *makespan = bw.m;
  if (info) {
    info->orders_fwd_total = tot_f; info->orders_bwd_total = tot_b;
    info->orders_fwd_tried = (int)of.size(); info->orders_bwd_tried = (int)ob.size();
    info->truncated = (tot_f > (long long)of.size() || tot_b > (long long)ob.size()) ? 1 : 0;
    info->refined = (int)refine.size();
  }
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
