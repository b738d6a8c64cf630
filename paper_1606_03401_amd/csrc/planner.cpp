// Host planner: the checkpoint-policy dynamic programs and the flattening of a policy into a
// linear schedule.
//
//   BPTT-HSM  Section 3.1, eq. 1-3, Algorithm 1      Q = y + C(t-y, m-1) + C(y, m),   1 <= y <  t
//   BPTT-ISM  Section 3.2, eq. 4-5                   Q = y + C(y-1, m) + C(t-y, m-1), 1 <= y <= t
//   BPTT-MSM  Sections 3.3-3.4, eq. 6-10             hidden push as HSM (1 unit) or internal push as
//                                                    ISM (alpha units; beta when y = 1)
//
// Ties of the argmin go to the smallest y (Algorithm 1 scans y upwards and replaces the
// incumbent only on a strictly smaller cost); between a hidden and an internal push of equal
// cost the hidden one is chosen.  Tables are solved column by column (one budget at a time,
// contiguous in t) and transposed into the row-major layout the ABI exposes.
//
// Flattening follows Algorithm 2 for hidden pushes, the four steps of Section 3.2 for internal
// pushes, and the constant-memory procedure of Section 3 when a single unit is left.  An
// internal state whose right-hand remainder is empty (y = t) is consumed by the next backward
// operation, so it is kept in the working core and not pushed.
//
// A policy need not come from the tables: Section 4.2 observes that any strategy inside the model
// -- Chen et al.'s two strategies of Section 2 in particular -- is a (possibly sub-optimal) policy
// of BPTT-MSM.  Such a policy is given as the list of decisions the flattening asks for, in the
// order it asks (a node, then its right sub-sequence, then its left one); the generators for the
// sqrt(t) and the recursive strategy produce that list.
#include <algorithm>
#include <cmath>
#include <cstring>
#include <new>
#include <string>

#include "common.h"

namespace mebptt {

static thread_local std::string g_last_error;

int set_error(int code, const char* fmt, ...) {
  char buf[512];
  va_list ap;
  va_start(ap, fmt);
  vsnprintf(buf, sizeof buf, fmt, ap);
  va_end(ap);
  g_last_error = buf;
  return code;
}

namespace {

constexpr int64_t INF = MEBPTT_COST_INF;

// min over y in [lo, hi] of  y + a[y - a_shift] + b_rev[-y]  with the smallest minimiser.
// a_shift is 0 (HSM: C(y, m)) or 1 (ISM: C(y-1, m)); b_rev points at b[t] so b_rev[-y] = b[t-y].
inline void first_argmin(const int64_t* a, int a_shift, const int64_t* b_rev, int lo, int hi, int64_t& best,
                         int& arg) {
  int64_t mn = INF;
  for (int y = lo; y <= hi; ++y) {
    int64_t c = (int64_t)y + a[y - a_shift] + b_rev[-y];
    mn = c < mn ? c : mn;
  }
  best = mn;
  arg = 0;
  if (mn >= INF) {
    best = INF;
    return;
  }
  for (int y = lo; y <= hi; ++y) {
    if ((int64_t)y + a[y - a_shift] + b_rev[-y] == mn) {
      arg = y;
      return;
    }
  }
}

// The O(t*m) route the appendix alludes to ("exploiting convexity in t").  If C(., m) is convex on
// the part already filled and C(., m-1) is convex, then Q(t, m, y) is convex in y (a sum of convex
// sequences), so a local minimum is the global one and the minimisers form an interval: the
// leftmost one is found by walking from the previous cell's split, in O(1) steps amortised.
// Convexity is not assumed: every column's second differences are checked as it is filled, and
// the first violation sends the rest of the table back to the full scan, so the result is always
// exactly the triple loop's (same cost, same leftmost split).
template <class QF>
inline void convex_first_argmin(QF Q, int lo, int hi, int start, int64_t& best, int& arg) {
  int y = start < lo ? lo : (start > hi ? hi : start);
  int64_t q = Q(y);
  while (y > lo) {   // ties go left
    int64_t ql = Q(y - 1);
    if (ql > q) break;
    --y;
    q = ql;
  }
  while (y < hi) {
    int64_t qr = Q(y + 1);
    if (qr >= q) break;
    ++y;
    q = qr;
  }
  best = q;
  arg = y;
}

// Second difference of a column at index i (needs i >= lo + 2).
inline bool convex_at(const std::vector<int64_t>& c, int i) { return c[i] - 2 * c[i - 1] + c[i - 2] >= 0; }

using Col64 = std::vector<std::vector<int64_t>>;
using Col32 = std::vector<std::vector<int32_t>>;

void alloc_cols(Col64& c, int t, int m, int64_t fill) { c.assign(m + 1, std::vector<int64_t>(t + 1, fill)); }
void alloc_cols(Col32& c, int t, int m) { c.assign(m + 1, std::vector<int32_t>(t + 1, 0)); }

template <class V, class T>
void to_row_major(const V& cols, int t, int m, std::vector<T>& out) {
  out.resize((size_t)(t + 1) * (m + 1));
  for (int mm = 0; mm <= m; ++mm)
    for (int tt = 0; tt <= t; ++tt) out[(size_t)tt * (m + 1) + mm] = cols[mm][tt];
}

void solve_hsm(int t, int m, Tables& T) {
  Col64 C;
  Col32 D;
  alloc_cols(C, t, m, INF);
  alloc_cols(D, t, m);
  for (int mm = 0; mm <= m; ++mm) C[mm][0] = 0;
  for (int tt = 1; tt <= t; ++tt) C[1][tt] = (int64_t)tt * (tt + 1) / 2;
  D[1][1] = 1;
  bool convex = true;   // every column so far (and the current one as far as filled) is convex on [0, .]
  for (int mm = 2; mm <= m; ++mm) {
    int plentiful = std::min(t, mm);
    for (int tt = 1; tt <= plentiful; ++tt) {
      C[mm][tt] = 2 * (int64_t)tt - 1;
      D[mm][tt] = 1;
    }
    const int64_t* cm = C[mm].data();
    const int64_t* cm1 = C[mm - 1].data();
    for (int tt = mm + 1; tt <= t; ++tt) {
      int64_t best;
      int arg;
      if (convex && tt > mm + 1) {
        auto Q = [&](int y) { return (int64_t)y + cm[y] + cm1[tt - y]; };
        convex_first_argmin(Q, 1, tt - 1, D[mm][tt - 1], best, arg);
      } else {
        first_argmin(cm, 0, cm1 + tt, 1, tt - 1, best, arg);
      }
      C[mm][tt] = best;
      D[mm][tt] = arg;
      if (convex && tt >= 2 && !convex_at(C[mm], tt)) convex = false;
    }
  }
  to_row_major(C, t, m, T.C);
  to_row_major(D, t, m, T.D);
}

void solve_ism(int t, int m, Tables& T) {
  Col64 C;
  Col32 D;
  alloc_cols(C, t, m, INF);
  alloc_cols(D, t, m);
  for (int mm = 0; mm <= m; ++mm) C[mm][0] = 0;
  bool convex = true;
  for (int mm = 1; mm <= m; ++mm) {
    const int64_t* cm = C[mm].data();
    const int64_t* cm1 = C[mm - 1].data();
    for (int tt = 1; tt <= t; ++tt) {
      int64_t best;
      int arg;
      // column 0 is infinite for t > 0, so the convexity argument starts with column 2
      if (mm == 1) {
        // a single slot: with C(t', 0) infinite for t' > 0, y = t is the only finite term of the scan
        best = (int64_t)tt + cm[tt - 1];
        arg = tt;
      } else if (convex && tt >= 2) {
        auto Q = [&](int y) { return (int64_t)y + cm[y - 1] + cm1[tt - y]; };
        convex_first_argmin(Q, 1, tt, D[mm][tt - 1], best, arg);
      } else {
        first_argmin(cm, 1, cm1 + tt, 1, tt, best, arg);
      }
      C[mm][tt] = best;
      D[mm][tt] = arg;
      if (convex && tt >= 2 && !convex_at(C[mm], tt)) convex = false;
    }
  }
  to_row_major(C, t, m, T.C);
  to_row_major(D, t, m, T.D);
}

void solve_msm(int t, int m, int alpha, int beta, Tables& T) {
  Col64 C, C1, C2;
  Col32 D1, D2;
  std::vector<std::vector<uint8_t>> Hc(m + 1, std::vector<uint8_t>(t + 1, 0));
  alloc_cols(C, t, m, INF);
  alloc_cols(C1, t, m, INF);
  alloc_cols(C2, t, m, INF);
  alloc_cols(D1, t, m);
  alloc_cols(D2, t, m);
  std::vector<int64_t> none(t + 1, INF);   // C(., m') for m' < 0
  for (int mm = 0; mm <= m; ++mm) C[mm][0] = 0;
  for (int tt = 1; tt <= t; ++tt) C[1][tt] = (int64_t)tt * (tt + 1) / 2;
  for (int mm = 1; mm <= m; ++mm) C[mm][1] = 1;
  for (int mm = 2; mm <= m; ++mm) {
    const int64_t* after_beta = (mm - beta >= 0) ? C[mm - beta].data() : none.data();
    const int64_t* after_alpha = (mm - alpha >= 0) ? C[mm - alpha].data() : none.data();
    for (int tt = 2; tt <= t; ++tt) {
      int64_t c1, c2;
      int d1, d2;
      first_argmin(C[mm].data(), 0, C[mm - 1].data() + tt, 1, tt - 1, c1, d1);
      // internal push: y = 1 takes beta units, y > 1 takes alpha units
      int64_t q_first = 1 + C[mm][0] + after_beta[tt - 1];
      first_argmin(C[mm].data(), 1, after_alpha + tt, 2, tt, c2, d2);
      if (q_first < INF && q_first <= c2) {
        c2 = q_first;
        d2 = 1;
      }
      C1[mm][tt] = c1;
      D1[mm][tt] = d1;
      C2[mm][tt] = c2;
      D2[mm][tt] = d2;
      if (c1 >= INF && c2 >= INF) continue;
      if (c1 <= c2) {
        C[mm][tt] = c1;
        Hc[mm][tt] = 1;
      } else {
        C[mm][tt] = c2;
        Hc[mm][tt] = 2;
      }
    }
  }
  to_row_major(C, t, m, T.C);
  to_row_major(C1, t, m, T.C1);
  to_row_major(C2, t, m, T.C2);
  to_row_major(D1, t, m, T.D1);
  to_row_major(D2, t, m, T.D2);
  to_row_major(Hc, t, m, T.Hc);
}

// ---- flattening ------------------------------------------------------------------------------

struct Work {
  enum { EXEC, BWD_AND_RELEASE, RELEASE } type;
  int32_t t, m, s, top;   // EXEC: sub-sequence length, budget, start index, location of its start state
  mebptt_op op;           // BWD_AND_RELEASE
  int32_t units;          // units handed back to the pool
};

inline int32_t transient(int parity) { return parity ? MEBPTT_LOC_T1 : MEBPTT_LOC_T0; }

class Flattener {
 public:
  Flattener(mebptt_plan_t& p, const std::vector<mebptt_decision>* list = nullptr) : p_(p), list_(list) {
    used_ = (p.kind == MEBPTT_ISM) ? 0 : 1;   // HSM/MSM: the start state h_0 occupies unit 0
    units_per_budget_ = (p.kind == MEBPTT_ISM) ? 4 : 1;
    capacity_ = (int64_t)p.m * units_per_budget_;
    peak_ = used_;
  }

  int run() {
    std::vector<Work> st;
    st.push_back(Work{Work::EXEC, p_.t, p_.m, 0, p_.kind == MEBPTT_ISM ? MEBPTT_LOC_INIT : 0, {}, 0});
    while (!st.empty()) {
      Work w = st.back();
      st.pop_back();
      if (w.type == Work::RELEASE) {
        used_ -= w.units;
        continue;
      }
      if (w.type == Work::BWD_AND_RELEASE) {
        emit(w.op);
        used_ -= w.units;
        continue;
      }
      int rc = exec(w, st);
      if (rc) return rc;
    }
    if (list_ && next_ != list_->size())
      return set_error(MEBPTT_EINVAL, "policy has %zu decisions, the schedule asked for %zu", list_->size(), next_);
    p_.peak = (int32_t)((peak_ + units_per_budget_ - 1) / units_per_budget_);
    return MEBPTT_OK;
  }

 private:
  void emit(const mebptt_op& op) {
    p_.ops.push_back(op);
    if (op.op == MEBPTT_OP_FWD_RUN)
      p_.forward_ops += op.count;
    else
      p_.backward_ops += 1;
  }

  // n forwards from `top` that end in the working core, then the backward of the last step.
  void forward_into_core_and_backward(int32_t s, int32_t n, int32_t top) {
    int32_t prev = n > 1 ? transient((n - 1) & 1) : MEBPTT_LOC_NONE;
    emit(mebptt_op{MEBPTT_OP_FWD_RUN, s + 1, n, top, MEBPTT_LOC_CORE, 1, prev});
    emit(mebptt_op{MEBPTT_OP_BWD, s + n, 1, n > 1 ? prev : top, MEBPTT_LOC_CORE, 0, MEBPTT_LOC_NONE});
  }

  int take(int32_t units) {
    used_ += units;
    if (used_ > capacity_)
      return list_ ? set_error(MEBPTT_EINFEASIBLE, "the policy needs more than the budget of %d units", p_.m)
                   : set_error(MEBPTT_EINVAL, "internal error: schedule exceeds the budget");
    peak_ = std::max(peak_, used_);
    return MEBPTT_OK;
  }

  int exec(const Work& w, std::vector<Work>& st) {
    const int32_t t = w.t, m = w.m, s = w.s, top = w.top;
    const Tables& T = p_.tab;
    if (t == 0) return MEBPTT_OK;
    bool internal;
    int32_t y;
    if (p_.kind == MEBPTT_ISM) {
      if (m < 1) return set_error(MEBPTT_EINFEASIBLE, "no slot left for a sub-sequence of length %d", t);
      internal = true;
      y = T.D[T.idx(t, m)];
    } else {
      if (t == 1) {   // base case of Section 3.1: forward and backward on the working core
        forward_into_core_and_backward(s, 1, top);
        return MEBPTT_OK;
      }
      if (m == 1) {   // constant-memory procedure of Section 3
        for (int32_t k = t; k >= 1; --k) forward_into_core_and_backward(s, k, top);
        return MEBPTT_OK;
      }
      if (list_) {   // caller-supplied policy: one decision per node with t >= 2 and m >= 2
        if (next_ >= list_->size())
          return set_error(MEBPTT_EINVAL, "policy ends after %zu decisions; node (t=%d, m=%d) needs one", next_, t, m);
        const mebptt_decision& d = (*list_)[next_++];
        if (d.store != MEBPTT_STORE_HIDDEN && d.store != MEBPTT_STORE_INTERNAL)
          return set_error(MEBPTT_EINVAL, "decision %zu: store must be 1 (hidden) or 2 (internal), got %d", next_ - 1, d.store);
        internal = d.store == MEBPTT_STORE_INTERNAL;
        y = d.y;
        if (y < 1 || (internal ? y > t : y >= t))
          return set_error(MEBPTT_EINVAL, "decision %zu: y=%d is outside the range of a sub-sequence of length %d", next_ - 1,
                           y, t);
        if (internal && y < t && m - (y == 1 ? p_.beta : p_.alpha) < 1)
          return set_error(MEBPTT_EINFEASIBLE, "decision %zu: an internal state does not fit into %d units", next_ - 1, m);
      } else if (p_.kind == MEBPTT_HSM) {
        internal = false;
        y = T.D[T.idx(t, m)];
      } else {
        uint8_t h = T.Hc[T.idx(t, m)];
        if (h == 0) return set_error(MEBPTT_EINFEASIBLE, "no feasible policy at (t=%d, m=%d)", t, m);
        internal = (h == 2);
        y = internal ? T.D2[T.idx(t, m)] : T.D1[T.idx(t, m)];
      }
    }
    if (!internal) {
      if (y < 1 || y >= t) return set_error(MEBPTT_EINVAL, "internal error: split %d outside [1,%d)", y, t);
      int32_t unit = (int32_t)used_;
      int rc = take(1);
      if (rc) return rc;
      int32_t prev = y > 1 ? transient((y - 1) & 1) : MEBPTT_LOC_NONE;
      emit(mebptt_op{MEBPTT_OP_FWD_RUN, s + 1, y, top, unit, 0, prev});
      st.push_back(Work{Work::EXEC, y, m, s, top, {}, 0});             // step 3: left part, full budget
      st.push_back(Work{Work::RELEASE, 0, 0, 0, 0, {}, 1});            // pop
      st.push_back(Work{Work::EXEC, t - y, m - 1, s + y, unit, {}, 0});   // step 2: right part
      return MEBPTT_OK;
    }
    if (y < 1 || y > t) return set_error(MEBPTT_EINVAL, "internal error: split %d outside [1,%d]", y, t);
    if (y == t) {   // nothing to the right: backward follows at once, no push
      forward_into_core_and_backward(s, y, top);
      st.push_back(Work{Work::EXEC, y - 1, m, s, top, {}, 0});
      return MEBPTT_OK;
    }
    int32_t units, cost_units;   // physical units taken; budget charged to the right part
    if (p_.kind == MEBPTT_ISM) {
      units = 4;
      cost_units = 1;
    } else {
      units = cost_units = (y == 1) ? p_.beta : p_.alpha;
    }
    int32_t base = (int32_t)used_;
    int rc = take(units);
    if (rc) return rc;
    // A full internal state keeps its input hidden state in its fourth unit: the forward run
    // writes state_{s+y-1} there directly.  With y = 1 the input state is the start state.
    bool own_input = (y > 1);
    if (own_input && units < 4)
      return set_error(MEBPTT_EINVAL, "an internal state with its input state needs 4 units (alpha=%d)", units);
    int32_t prev = own_input ? base + 3 : MEBPTT_LOC_NONE;
    emit(mebptt_op{MEBPTT_OP_FWD_RUN, s + 1, y, top, base, 1, prev});
    mebptt_op bwd{MEBPTT_OP_BWD, s + y, 1, own_input ? base + 3 : top, base, 0, MEBPTT_LOC_NONE};
    st.push_back(Work{Work::EXEC, y - 1, m, s, top, {}, 0});                        // step 4: left part
    st.push_back(Work{Work::BWD_AND_RELEASE, 0, 0, 0, 0, bwd, units});              // step 3 + release
    st.push_back(Work{Work::EXEC, t - y, m - cost_units, s + y, base, {}, 0});      // step 2: right part
    return MEBPTT_OK;
  }

  mebptt_plan_t& p_;
  const std::vector<mebptt_decision>* list_;
  size_t next_ = 0;
  int64_t used_, peak_, capacity_;
  int32_t units_per_budget_;
};

// ---- Chen et al.'s strategies as decision lists (Section 2; Section 4.2) -----------------------

inline int32_t ceil_div(int32_t a, int32_t b) { return (a + b - 1) / b; }

// A part that is run with every internal state memorised: each state is pushed right after the
// step that made it (y = 1, beta units: its input state is the entry below).
void chen_keep_all(int32_t n, std::vector<mebptt_decision>& out) {
  for (int32_t i = 0; i + 1 < n; ++i) out.push_back(mebptt_decision{MEBPTT_STORE_INTERNAL, 1});
}

// sqrt(t): ceil(sqrt(t)) parts of equal length L, the hidden state memorised at every cut, each
// part then (re)run keeping all of its internal states.  The cuts nest to the right, so their
// decisions come first, then the last part, then one full part per cut while unwinding.
void chen_sqrt_decisions(int32_t t, std::vector<mebptt_decision>& out) {
  int32_t k = (int32_t)std::ceil(std::sqrt((double)t));
  while ((int64_t)k * k < t) ++k;
  while (k > 1 && (int64_t)(k - 1) * (k - 1) >= t) --k;
  const int32_t L = ceil_div(t, k), ncut = ceil_div(t, L) - 1;
  for (int32_t j = 0; j < ncut; ++j) out.push_back(mebptt_decision{MEBPTT_STORE_HIDDEN, L});
  chen_keep_all(t - L * ncut, out);
  for (int32_t j = 0; j < ncut; ++j) chen_keep_all(L, out);
}

// recursive, k memorised hidden states per level: a sub-sequence of length n is cut into
// min(k+1, n) parts of equal length, each part treated the same way until its length is 1.
void chen_recursive_decisions(int32_t n, int32_t k, std::vector<mebptt_decision>& out) {
  if (n <= 1) return;
  const int32_t parts = (int32_t)std::min<int64_t>((int64_t)k + 1, n);
  const int32_t L = ceil_div(n, parts), ncut = ceil_div(n, L) - 1;
  for (int32_t j = 0; j < ncut; ++j) out.push_back(mebptt_decision{MEBPTT_STORE_HIDDEN, L});
  chen_recursive_decisions(n - L * ncut, k, out);
  for (int32_t j = 0; j < ncut; ++j) chen_recursive_decisions(L, k, out);
}

int check_policy_args(int32_t t, int32_t alpha, int32_t beta, mebptt_plan_t** out) {
  if (!out) return set_error(MEBPTT_EINVAL, "out is NULL");
  *out = nullptr;
  if (t < 1) return set_error(MEBPTT_EINVAL, "t must be >= 1 (got %d)", t);
  if (alpha < 4 || beta < 3 || beta > alpha)
    return set_error(MEBPTT_EINVAL, "a schedule needs alpha >= 4 and 3 <= beta <= alpha (got %d, %d)", alpha, beta);
  return MEBPTT_OK;
}

// Flattens `list` for (t, m) in the MSM protocol.  m <= 0: the budget becomes what the policy needs.
int plan_from_list(int32_t t, int32_t m, int32_t alpha, int32_t beta, const std::vector<mebptt_decision>& list,
                   mebptt_plan_t** out) {
  for (int pass = (m > 0 ? 1 : 0); pass < 2; ++pass) {
    mebptt_plan_t* p = new (std::nothrow) mebptt_plan_t;
    if (!p) return set_error(MEBPTT_ENOMEM_HOST, "out of host memory");
    p->t = t;
    p->m = pass ? m : INT32_MAX / 8;   // sizing pass: no limit, the peak becomes the budget
    p->kind = MEBPTT_MSM;
    p->alpha = alpha;
    p->beta = beta;
    p->from_policy = true;
    int rc;
    try {
      Flattener f(*p, &list);
      rc = f.run();
    } catch (const std::bad_alloc&) {
      rc = set_error(MEBPTT_ENOMEM_HOST, "out of host memory");
    }
    if (rc) {
      delete p;
      return rc;
    }
    if (pass) {
      *out = p;
      return MEBPTT_OK;
    }
    m = p->peak;
    delete p;
  }
  return MEBPTT_OK;
}

}  // namespace
}  // namespace mebptt

using namespace mebptt;

extern "C" {

int mebptt_plan(int32_t t, int32_t m, int32_t kind, int32_t alpha, int32_t beta, mebptt_plan_t** out) {
  if (!out) return set_error(MEBPTT_EINVAL, "out is NULL");
  *out = nullptr;
  if (t < 1) return set_error(MEBPTT_EINVAL, "t must be >= 1 (got %d)", t);
  if (m < 1) return set_error(MEBPTT_EINVAL, "m must be >= 1 (got %d)", m);
  if (kind != MEBPTT_HSM && kind != MEBPTT_ISM && kind != MEBPTT_MSM)
    return set_error(MEBPTT_EINVAL, "unknown kind %d", kind);
  if (kind == MEBPTT_MSM) {
    if (alpha < 2) return set_error(MEBPTT_EINVAL, "alpha must be an integer >= 2 (got %d)", alpha);
    if (beta < 1 || beta > alpha) return set_error(MEBPTT_EINVAL, "beta must be in [1, alpha] (got %d)", beta);
  }
  if ((int64_t)(t + 1) * (int64_t)(m + 1) > ((int64_t)1 << 31))
    return set_error(MEBPTT_ENOMEM_HOST, "tables of %d x %d cells are too large", t + 1, m + 1);
  mebptt_plan_t* p = new (std::nothrow) mebptt_plan_t;
  if (!p) return set_error(MEBPTT_ENOMEM_HOST, "out of host memory");
  try {
    p->t = t;
    p->m = m;
    p->kind = kind;
    p->alpha = kind == MEBPTT_MSM ? alpha : 0;
    p->beta = kind == MEBPTT_MSM ? beta : 0;
    p->tab.t = t;
    p->tab.m = m;
    if (kind == MEBPTT_HSM)
      solve_hsm(t, m, p->tab);
    else if (kind == MEBPTT_ISM)
      solve_ism(t, m, p->tab);
    else
      solve_msm(t, m, alpha, beta, p->tab);
    if (p->tab.C[p->tab.idx(t, m)] >= INF) {
      delete p;
      return set_error(MEBPTT_EINFEASIBLE, "C(%d, %d) is infinite: the budget cannot hold the sequence", t, m);
    }
    if (kind == MEBPTT_MSM && !(alpha >= 4 && beta >= 3)) {
      // tables only: an LSTM internal state needs 4 units (3 without its input state), so no
      // schedule exists for smaller state sizes.  Larger ones leave the extra units unused.
      *out = p;
      return MEBPTT_OK;
    }
    Flattener f(*p);
    int rc = f.run();
    if (rc) {
      delete p;
      return rc;
    }
  } catch (const std::bad_alloc&) {
    delete p;
    return set_error(MEBPTT_ENOMEM_HOST, "out of host memory");
  }
  *out = p;
  return MEBPTT_OK;
}

int mebptt_plan_from_policy(int32_t t, int32_t m, int32_t alpha, int32_t beta, const mebptt_decision* decisions,
                            size_t n, mebptt_plan_t** out) {
  int rc = check_policy_args(t, alpha, beta, out);
  if (rc) return rc;
  if (m < 1) return set_error(MEBPTT_EINVAL, "m must be >= 1 (got %d)", m);
  if (n && !decisions) return set_error(MEBPTT_EINVAL, "decisions is NULL");
  try {
    std::vector<mebptt_decision> list(decisions, decisions + n);
    return plan_from_list(t, m, alpha, beta, list, out);
  } catch (const std::bad_alloc&) {
    return set_error(MEBPTT_ENOMEM_HOST, "out of host memory");
  }
}

int mebptt_plan_chen_sqrt(int32_t t, int32_t alpha, int32_t beta, mebptt_plan_t** out) {
  int rc = check_policy_args(t, alpha, beta, out);
  if (rc) return rc;
  try {
    std::vector<mebptt_decision> list;
    chen_sqrt_decisions(t, list);
    return plan_from_list(t, 0, alpha, beta, list, out);
  } catch (const std::bad_alloc&) {
    return set_error(MEBPTT_ENOMEM_HOST, "out of host memory");
  }
}

int mebptt_plan_chen_recursive(int32_t t, int32_t k, int32_t alpha, int32_t beta, mebptt_plan_t** out) {
  int rc = check_policy_args(t, alpha, beta, out);
  if (rc) return rc;
  if (k < 1) return set_error(MEBPTT_EINVAL, "k must be >= 1 (got %d)", k);
  try {
    std::vector<mebptt_decision> list;
    chen_recursive_decisions(t, k, list);
    return plan_from_list(t, 0, alpha, beta, list, out);
  } catch (const std::bad_alloc&) {
    return set_error(MEBPTT_ENOMEM_HOST, "out of host memory");
  }
}

void mebptt_plan_free(mebptt_plan_t* plan) { delete plan; }

const int64_t* mebptt_plan_cost(const mebptt_plan_t* p, int32_t which) {
  if (!p || p->from_policy) return nullptr;
  if (which == 0) return p->tab.C.data();
  if (p->kind != MEBPTT_MSM) return nullptr;
  if (which == 1) return p->tab.C1.data();
  if (which == 2) return p->tab.C2.data();
  return nullptr;
}

const int32_t* mebptt_plan_split(const mebptt_plan_t* p, int32_t which) {
  if (!p || p->from_policy) return nullptr;
  if (p->kind != MEBPTT_MSM) return which == 0 ? p->tab.D.data() : nullptr;
  if (which == 1) return p->tab.D1.data();
  if (which == 2) return p->tab.D2.data();
  return nullptr;
}

const uint8_t* mebptt_plan_choice(const mebptt_plan_t* p) {
  return (p && p->kind == MEBPTT_MSM && !p->from_policy) ? p->tab.Hc.data() : nullptr;
}

int32_t mebptt_plan_length(const mebptt_plan_t* p) { return p ? p->t : 0; }
int32_t mebptt_plan_budget(const mebptt_plan_t* p) { return p ? p->m : 0; }
int32_t mebptt_plan_kind(const mebptt_plan_t* p) { return p ? p->kind : -1; }
int64_t mebptt_plan_forward_ops(const mebptt_plan_t* p) { return p ? p->forward_ops : 0; }
int32_t mebptt_plan_peak(const mebptt_plan_t* p) { return p ? p->peak : 0; }

const mebptt_op* mebptt_plan_schedule(const mebptt_plan_t* p, size_t* n) {
  if (n) *n = p ? p->ops.size() : 0;
  return p ? p->ops.data() : nullptr;
}

const char* mebptt_last_error(void) { return g_last_error.c_str(); }

const char* mebptt_version(void) { return "mebptt 0.1 (gfx950)"; }

}  // extern "C"
