// Host planner for a linear chain of non-homogeneous layers (appendix "Generalizing to deep
// feed-forward networks").
//
// Layer i (1-based) has a forward cost u_i, an output of s_i memory units and needs p_i units of
// working memory while its forward or backward operation runs.  C(t, m, x) is the cost of
// back-propagating through layers x+1 .. x+t when the input of layer x+1 is available and m units
// are free:
//
//   Q(t, m, y, x) = U(x, y) + K(x, y, m) + C(t - y, m - s_{x+y}, x + y) + C(y, m, x),   1 <= y < t
//   C(t, m, x)    = min_y Q,   D(t, m, x) = the smallest minimising y
//
// with U the forward cost of y layers above the cut x and K infinite when their working memory
// does not fit.  Readings of the appendix's boundary conditions: C(0, ., .) = 0; one layer costs
// u if its working memory fits; at every node the sub-chain may also be processed without
// memorising anything (re-run from its input before every backward step: the appendix's cost for
// "no extra memory left"), recorded as D = 0; a tie goes to the memorisation.  The network input is
// always available and not counted.  With u = 1, s = 1, p = 0 this is BPTT-HSM with the start
// state outside the budget.
//
// The table is three-dimensional (the appendix notes it), stored as [x][t][m] for x + t <= n.
// The schedule is flattened the way the appendix's last paragraph executes the policy.
#include <algorithm>
#include <cstdint>
#include <new>
#include <vector>

#include "common.h"

using namespace mebptt;

struct mebptt_chain_plan_s {
  int32_t n = 0, m = 0;
  std::vector<mebptt_layer> layers;
  std::vector<int64_t> prefix;       // prefix[i] = u_1 + ... + u_i
  std::vector<size_t> base;          // base[x] = index of cell (x, t = 0, m = 0)
  std::vector<int64_t> C;
  std::vector<int32_t> D;
  std::vector<mebptt_chain_op> ops;
  int64_t forward_cost = 0;
  int32_t peak = 0;

  size_t idx(int32_t t, int32_t mm, int32_t x) const { return base[x] + (size_t)t * (m + 1) + mm; }
  int64_t U(int32_t x, int32_t y) const { return prefix[x + y] - prefix[x]; }
  int64_t cost(int32_t t, int32_t mm, int32_t x) const {
    if (mm < 0) return MEBPTT_COST_INF;
    return C[idx(t, mm, x)];
  }
};

namespace {

constexpr int64_t INF = MEBPTT_COST_INF;

void solve(mebptt_chain_plan_s& p) {
  const int32_t n = p.n, m = p.m;
  p.base.resize(n + 1);
  size_t cells = 0;
  for (int32_t x = 0; x <= n; ++x) {
    p.base[x] = cells;
    cells += (size_t)(n - x + 1) * (m + 1);
  }
  p.C.assign(cells, INF);
  p.D.assign(cells, 0);
  for (int32_t x = 0; x <= n; ++x)
    for (int32_t mm = 0; mm <= m; ++mm) p.C[p.idx(0, mm, x)] = 0;
  // Sub-chains by length: a cell needs shorter sub-chains only.
  std::vector<int32_t> pmax(n + 1);   // pmax[y] = P(x, y) for the current x
  std::vector<int64_t> rerun(n + 1);  // rerun[t] = U(x,1) + ... + U(x,t)
  for (int32_t t = 1; t <= n; ++t) {
    for (int32_t x = 0; x + t <= n; ++x) {
      pmax[0] = 0;
      rerun[0] = 0;
      for (int32_t y = 1; y <= t; ++y) {
        pmax[y] = std::max(pmax[y - 1], p.layers[x + y - 1].work_units);
        rerun[y] = rerun[y - 1] + p.U(x, y);
      }
      for (int32_t mm = 0; mm <= m; ++mm) {
        int64_t best = INF;
        int32_t arg = 0;
        if (t == 1) {
          if (pmax[1] <= mm) best = p.layers[x].cost;
        } else {
          if (pmax[t] <= mm) best = rerun[t];
          for (int32_t y = 1; y < t; ++y) {
            if (pmax[y] > mm) break;   // working memory only grows with y
            const int32_t rest = mm - p.layers[x + y - 1].state_units;
            if (rest < 0) continue;
            const int64_t right = p.C[p.idx(t - y, rest, x + y)];
            const int64_t left = p.C[p.idx(y, mm, x)];
            if (right >= INF || left >= INF) continue;
            const int64_t q = p.U(x, y) + right + left;
            if (q < best || (q == best && arg == 0)) {
              best = q;
              arg = y;
            }
          }
        }
        p.C[p.idx(t, mm, x)] = best;
        p.D[p.idx(t, mm, x)] = arg;
      }
    }
  }
}

// Flattening with an explicit work stack.  Memorised outputs are stacked in a pool of m units,
// each at the unit offset at which it was pushed.
struct Work {
  enum { EXEC, RELEASE } type;
  int32_t t, mm, x, src;   // EXEC: sub-chain and the location of its input
  int32_t units;           // RELEASE
};

int flatten(mebptt_chain_plan_s& p) {
  std::vector<Work> st;
  int64_t used = 0, peak = 0;
  auto work = [&](int32_t first, int32_t count) {   // working memory of layers first .. first+count-1
    int32_t w = 0;
    for (int32_t i = 0; i < count; ++i) w = std::max(w, p.layers[first - 1 + i].work_units);
    peak = std::max(peak, used + w);
  };
  st.push_back(Work{Work::EXEC, p.n, p.m, 0, MEBPTT_CHAIN_INPUT, 0});
  while (!st.empty()) {
    const Work w = st.back();
    st.pop_back();
    if (w.type == Work::RELEASE) {
      used -= w.units;
      continue;
    }
    const int32_t t = w.t, mm = w.mm, x = w.x;
    if (t == 0) continue;
    if (t == 1) {
      p.ops.push_back(mebptt_chain_op{MEBPTT_CHAIN_FORWARD, x + 1, 1, w.src, MEBPTT_CHAIN_WORKING});
      p.ops.push_back(mebptt_chain_op{MEBPTT_CHAIN_BACKWARD, x + 1, 1, w.src, MEBPTT_CHAIN_WORKING});
      p.forward_cost += p.layers[x].cost;
      work(x + 1, 1);
      continue;
    }
    const int32_t y = p.D[p.idx(t, mm, x)];
    if (y == 0) {   // no memorisation: re-run from the sub-chain's input before every backward step
      for (int32_t k = t; k >= 1; --k) {
        p.ops.push_back(mebptt_chain_op{MEBPTT_CHAIN_FORWARD, x + 1, k, w.src, MEBPTT_CHAIN_WORKING});
        p.ops.push_back(mebptt_chain_op{MEBPTT_CHAIN_BACKWARD, x + k, 1, k > 1 ? MEBPTT_CHAIN_WORKING : w.src,
                                        MEBPTT_CHAIN_WORKING});
        p.forward_cost += p.U(x, k);
        work(x + 1, k);
      }
      continue;
    }
    const int32_t units = p.layers[x + y - 1].state_units;
    const int32_t at = (int32_t)used;
    p.ops.push_back(mebptt_chain_op{MEBPTT_CHAIN_FORWARD, x + 1, y, w.src, at});
    p.forward_cost += p.U(x, y);
    work(x + 1, y);
    used += units;
    peak = std::max(peak, used);
    if (used > p.m) return set_error(MEBPTT_EINVAL, "internal error: chain schedule exceeds the budget");
    st.push_back(Work{Work::EXEC, y, mm, x, w.src, 0});                    // left part, full budget
    st.push_back(Work{Work::RELEASE, 0, 0, 0, 0, units});                  // the memorised output is dropped
    st.push_back(Work{Work::EXEC, t - y, mm - units, x + y, at, 0});       // right part first
  }
  p.peak = (int32_t)peak;
  return MEBPTT_OK;
}

}  // namespace

extern "C" {

int mebptt_chain_plan(const mebptt_layer* layers, int32_t n, int32_t m, mebptt_chain_plan_t** out) {
  if (!out) return set_error(MEBPTT_EINVAL, "out is NULL");
  *out = nullptr;
  if (!layers || n < 1) return set_error(MEBPTT_EINVAL, "a chain needs at least one layer");
  if (m < 0) return set_error(MEBPTT_EINVAL, "m must be >= 0 (got %d)", m);
  for (int32_t i = 0; i < n; ++i)
    if (layers[i].cost < 1 || layers[i].state_units < 1 || layers[i].work_units < 0)
      return set_error(MEBPTT_EINVAL, "layer %d: cost and state size must be >= 1, working size >= 0", i + 1);
  if ((double)(n + 1) * (n + 2) / 2 * ((double)m + 1) > (double)((int64_t)1 << 28))
    return set_error(MEBPTT_ENOMEM_HOST, "a table of %d layers x %d units is too large", n, m);
  mebptt_chain_plan_s* p = new (std::nothrow) mebptt_chain_plan_s;
  if (!p) return set_error(MEBPTT_ENOMEM_HOST, "out of host memory");
  int rc = MEBPTT_OK;
  try {
    p->n = n;
    p->m = m;
    p->layers.assign(layers, layers + n);
    p->prefix.assign(n + 1, 0);
    for (int32_t i = 0; i < n; ++i) p->prefix[i + 1] = p->prefix[i] + layers[i].cost;
    solve(*p);
    if (p->C[p->idx(n, m, 0)] >= INF)
      rc = set_error(MEBPTT_EINFEASIBLE, "C(%d, %d, 0) is infinite: the chain does not fit into %d units", n, m, m);
    else
      rc = flatten(*p);
  } catch (const std::bad_alloc&) {
    rc = set_error(MEBPTT_ENOMEM_HOST, "out of host memory");
  }
  if (rc) {
    delete p;
    return rc;
  }
  *out = p;
  return MEBPTT_OK;
}

void mebptt_chain_plan_free(mebptt_chain_plan_t* plan) { delete plan; }

int64_t mebptt_chain_cost(const mebptt_chain_plan_t* p, int32_t t, int32_t m, int32_t x) {
  if (!p || t < 0 || x < 0 || x + t > p->n || m > p->m) return MEBPTT_COST_INF;
  return p->cost(t, m, x);
}

int32_t mebptt_chain_split(const mebptt_chain_plan_t* p, int32_t t, int32_t m, int32_t x) {
  if (!p || t < 0 || x < 0 || x + t > p->n || m > p->m || m < 0) return 0;
  return p->D[p->idx(t, m, x)];
}

int64_t mebptt_chain_plan_forward_cost(const mebptt_chain_plan_t* p) { return p ? p->forward_cost : 0; }
int32_t mebptt_chain_plan_peak(const mebptt_chain_plan_t* p) { return p ? p->peak : 0; }

const mebptt_layer* mebptt_chain_plan_layers(const mebptt_chain_plan_t* p, int32_t* n) {
  if (n) *n = p ? p->n : 0;
  return p ? p->layers.data() : nullptr;
}

const mebptt_chain_op* mebptt_chain_plan_schedule(const mebptt_chain_plan_t* p, size_t* n) {
  if (n) *n = p ? p->ops.size() : 0;
  return p ? p->ops.data() : nullptr;
}

}  // extern "C"
