// ILPSolve of Algorithm 3 on the host: the integer program of Section 3.2 ("Dynamic quantization configurations")
//     minimise   sum_i error[i][c_i]     subject to   sum_i storage[i][c_i] <= budget,   one configuration c_i per matrix
// is a multiple-choice knapsack.  The paper hands it to an external solver; this is a self-contained exact method:
// per matrix the dominated configurations are dropped and the lower convex hull of (storage, error) is built; the
// linear relaxation is then solved greedily by taking hull segments in order of error removed per bit (at most one
// matrix ends up fractional), which gives a lower bound and, by rounding down, a feasible assignment; depth-first
// branch and bound on the fractional matrix closes the gap.  Every node costs one pass over the sorted segments.
#include <algorithm>
#include <cmath>
#include <limits>
#include <vector>

#include "lq_internal.h"

namespace lq {
namespace {

struct Option { double s, e; int cfg; };
struct Segment { double slope, ds, de; int item, to; };   // hull step of `item` that ends at hull point `to`

struct Problem {
  int n = 0;
  double budget = 0;
  std::vector<std::vector<Option>> opts;    // non-dominated, storage increasing, error strictly decreasing
  std::vector<std::vector<int>> hull;       // indices into opts[i]: lower convex hull, hull[i][0] = cheapest
  std::vector<Segment> segs;                // all hull steps, steepest (most error removed per bit) first
  // search state
  std::vector<int> fixed;                   // option index per item, -1 = free
  std::vector<int> best;
  double best_err = std::numeric_limits<double>::infinity();
  long nodes = 0, node_limit = 0;
  bool complete = true;
};

struct Relaxed {
  double bound;        // value of the linear relaxation (infinity when infeasible)
  double err, used;    // value and storage of the rounded-down assignment
  int frac_item;       // matrix whose hull step was cut by the budget, -1 if none
  std::vector<int> pick;
};

// Linear relaxation over the free items with the fixed ones charged first.
Relaxed relax(const Problem& p) {
  Relaxed r;
  r.pick.assign(p.n, 0);
  r.frac_item = -1;
  double err = 0, used = 0;
  for (int i = 0; i < p.n; ++i) {
    const int o = p.fixed[i] >= 0 ? p.fixed[i] : p.hull[i][0];
    r.pick[i] = o;
    err += p.opts[i][o].e;
    used += p.opts[i][o].s;
  }
  if (used > p.budget) { r.bound = std::numeric_limits<double>::infinity(); r.err = r.bound; r.used = used; return r; }
  double bound = err;
  bool cut = false;
  std::vector<char> blocked(p.n, 0);         // an item whose step did not fit takes no later step
  for (const Segment& g : p.segs) {
    if (p.fixed[g.item] >= 0 || blocked[g.item]) continue;
    if (used + g.ds <= p.budget) {
      used += g.ds; err += g.de;
      if (!cut) bound = err;
      r.pick[g.item] = p.hull[g.item][g.to];
    } else {
      if (!cut) {                            // first step that does not fit: the relaxation takes a fraction of it
        bound = err + g.de * (p.budget - used) / g.ds;
        r.frac_item = g.item;
        cut = true;
      }
      blocked[g.item] = 1;
    }
  }
  r.bound = bound; r.err = err; r.used = used;
  return r;
}

void search(Problem& p) {
  if (p.node_limit && p.nodes >= p.node_limit) { p.complete = false; return; }
  ++p.nodes;
  const Relaxed r = relax(p);
  if (!(r.bound < p.best_err)) return;                      // infeasible or cannot improve
  if (r.err < p.best_err) { p.best_err = r.err; p.best = r.pick; }
  if (r.frac_item < 0) return;                              // relaxation is integral: this subtree is solved
  const int i = r.frac_item;
  // children: every remaining option of the fractional matrix, the rounded-down choice first, then by storage
  std::vector<int> order;
  order.push_back(r.pick[i]);
  for (int o = 0; o < (int)p.opts[i].size(); ++o) if (o != r.pick[i]) order.push_back(o);
  for (int o : order) {
    p.fixed[i] = o;
    search(p);
  }
  p.fixed[i] = -1;
}

}  // namespace
}  // namespace lq

using namespace lq;

extern "C" int lq_assign_configs(const double* err, const double* storage, int n_matrices, int n_cfgs,
                                 double budget_bits, int64_t node_limit, int32_t* choice, double* total_err,
                                 double* total_storage, double* lower_bound) {
  if (!err || !storage || !choice) return LQ_ERR_NULL;
  if (n_matrices < 1 || n_cfgs < 1 || node_limit < 0 || !(budget_bits >= 0)) return LQ_ERR_ARG;
  Problem p;
  p.n = n_matrices;
  p.budget = budget_bits;
  p.node_limit = (long)node_limit;
  p.opts.resize(p.n);
  p.hull.resize(p.n);
  for (int i = 0; i < p.n; ++i) {
    std::vector<Option> all(n_cfgs);
    for (int c = 0; c < n_cfgs; ++c) {
      const double s = storage[(size_t)i * n_cfgs + c], e = err[(size_t)i * n_cfgs + c];
      if (!std::isfinite(s) || !std::isfinite(e) || s < 0 || e < 0) return LQ_ERR_ARG;
      all[c] = Option{s, e, c};
    }
    // cheapest first; among equals the smaller error, then the smaller index (deterministic)
    std::sort(all.begin(), all.end(), [](const Option& a, const Option& b) {
      if (a.s != b.s) return a.s < b.s;
      if (a.e != b.e) return a.e < b.e;
      return a.cfg < b.cfg;
    });
    for (const Option& o : all)
      if (p.opts[i].empty() || o.e < p.opts[i].back().e) p.opts[i].push_back(o);     // not dominated
    // lower convex hull: slopes (error removed per bit) must decrease in magnitude from step to step
    std::vector<int>& h = p.hull[i];
    for (int o = 0; o < (int)p.opts[i].size(); ++o) {
      while (h.size() >= 2) {
        const Option& a = p.opts[i][h[h.size() - 2]];
        const Option& b = p.opts[i][h.back()];
        const Option& c = p.opts[i][o];
        // b lies on or above the chord a-c  <=>  (b.e - a.e) * (c.s - a.s) >= (c.e - a.e) * (b.s - a.s)
        if ((b.e - a.e) * (c.s - a.s) >= (c.e - a.e) * (b.s - a.s)) h.pop_back();
        else break;
      }
      h.push_back(o);
    }
    for (int t = 1; t < (int)h.size(); ++t) {
      const Option& a = p.opts[i][h[t - 1]];
      const Option& b = p.opts[i][h[t]];
      p.segs.push_back(Segment{(b.e - a.e) / (b.s - a.s), b.s - a.s, b.e - a.e, i, t});
    }
  }
  std::stable_sort(p.segs.begin(), p.segs.end(), [](const Segment& a, const Segment& b) {
    if (a.slope != b.slope) return a.slope < b.slope;       // most negative first
    if (a.item != b.item) return a.item < b.item;
    return a.to < b.to;
  });
  p.fixed.assign(p.n, -1);
  const Relaxed root = relax(p);
  if (!std::isfinite(root.bound)) return LQ_ERR_ARG;        // even the cheapest configurations exceed the budget
  search(p);
  double te = 0, ts = 0;
  for (int i = 0; i < p.n; ++i) {
    const Option& o = p.opts[i][p.best[i]];
    choice[i] = o.cfg;
    te += o.e; ts += o.s;
  }
  if (total_err) *total_err = te;
  if (total_storage) *total_storage = ts;
  if (lower_bound) *lower_bound = p.complete ? te : std::min(te, root.bound);
  return LQ_OK;
}
