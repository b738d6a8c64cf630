// Executor: walks the flat schedule of a plan and enqueues the HIP kernels of one gradient step
// (Algorithm 2 for hidden-state pushes, Section 3.2's four steps for internal-state pushes).
//
// Memory outside the slot budget (the "single RNN core available for intermediate
// calculations" of Section 3.1, plus bounded staging) lives in the caller's workspace:
//   operand copies of the weights | transient states T0, T1 | working core (3 units, held twice so
//   that the forward step of the next backward operation can be computed while the previous one
//   is still being back-propagated) | copy of (h0, c0) | running dc | two chunk buffers each of
//   dG, dG^T and [x ; h_prev]^T.
// The weight gradient is accumulated once per chunk of CH consecutive time steps.  Chunks are
// aligned to absolute step numbers, so the summation order of dW depends only on t -- never on
// the budget or the policy -- and gradients are bit-identical for every budget.
#include <hip/hip_runtime.h>

#include <cstring>
#include <mutex>
#include <vector>

#include "common.h"
#include "kernels.h"

using namespace mebptt;

namespace {

constexpr size_t ALIGN = 256;
inline size_t align_up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }

struct Workspace {
  size_t Wp, bp, WTh, WTx, state, dWacc, dc, dG[2], dGT[2], aT[2], total;
};

Workspace layout(const Dims& d) {
  Workspace w{};
  const size_t op = d.op_bytes();
  const size_t unit = d.unit * sizeof(float);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t o = off;
    off = align_up(off + bytes);
    return o;
  };
  w.Wp = take((size_t)d.G4 * d.KP * op);
  w.bp = take((size_t)d.G4 * sizeof(float));
  w.WTh = take((size_t)d.HP * d.G4 * op);
  w.WTx = take((size_t)d.NX * d.G4 * op);
  w.state = take(9 * unit);   // T0 | T1 | core A (3 units) | copy of (h0,c0) | core B (3 units)
  w.dWacc = take(wgrad_accumulator_bytes(d));
  w.dc = take((size_t)d.B * d.H * sizeof(float));
  for (int i = 0; i < 2; ++i) w.dG[i] = take((size_t)d.CH * d.BP * d.G4 * op);
  for (int i = 0; i < 2; ++i) w.dGT[i] = take((size_t)d.G4 * d.KC * op);
  for (int i = 0; i < 2; ++i) w.aT[i] = take((size_t)d.NA * d.KC * op);
  w.total = off;
  return w;
}

int check_desc(const mebptt_lstm_desc* desc) {
  if (!desc) return set_error(MEBPTT_EINVAL, "desc is NULL");
  if (desc->B < 1 || desc->I < 1 || desc->H < 1 || desc->t < 1)
    return set_error(MEBPTT_EINVAL, "B, I, H, t must be >= 1 (got %d, %d, %d, %d)", desc->B, desc->I, desc->H, desc->t);
  if (desc->gemm_dtype != 0 && desc->gemm_dtype != 1)
    return set_error(MEBPTT_EINVAL, "gemm_dtype must be 0 (fp32) or 1 (bf16)");
  if (desc->loss != 0 && desc->loss != 1) return set_error(MEBPTT_EINVAL, "loss must be 0 or 1");
  if (desc->cell != MEBPTT_CELL_LSTM && desc->cell != MEBPTT_CELL_GRU)
    return set_error(MEBPTT_EINVAL, "cell must be 0 (LSTM) or 1 (GRU) (got %d)", desc->cell);
  if (desc->loss == 0 && (desc->dy_first_step < 1 || desc->dy_first_step > desc->t))
    return set_error(MEBPTT_EINVAL, "dy_first_step must be in [1, t] (got %d)", desc->dy_first_step);
  if ((int64_t)desc->B * desc->H > (int64_t)1 << 28 || (int64_t)desc->H * 4 * ((int64_t)desc->I + desc->H) > (int64_t)1 << 31)
    return set_error(MEBPTT_EINVAL, "shape too large");
  return MEBPTT_OK;
}

inline bool misaligned(const void* p, size_t a) { return (reinterpret_cast<uintptr_t>(p) & (a - 1)) != 0; }

// ---- optional event sampling (measurement hook) ------------------------------------------------
struct Sample {
  int cls;
  hipEvent_t start, stop;
  int64_t launches;   // kernel launches between the two events
};
struct Profiler {
  int every_n = 0;
  bool in_run = false;   // inside a bracketed forward run: no per-launch brackets
  int64_t launches[MEBPTT_K_CLASSES] = {};
  std::vector<Sample> pending;
  std::vector<Sample> runs;   // whole forward runs, one event pair around many launches
  std::vector<hipEvent_t> pool;
  hipEvent_t get() {
    if (!pool.empty()) {
      hipEvent_t e = pool.back();
      pool.pop_back();
      return e;
    }
    hipEvent_t e = nullptr;
    if (hipEventCreate(&e) != hipSuccess) return nullptr;
    return e;
  }
};
Profiler g_prof;

// Brackets one launch with events when it falls on the sampling grid.
template <class F>
hipError_t timed(int cls, hipStream_t st, F&& launch) {
  Profiler& p = g_prof;
  if (p.every_n <= 0) return launch();
  const bool sample = (p.launches[cls]++ % p.every_n) == 0 && p.pending.size() < 200000 && !p.in_run;
  if (!sample) return launch();
  Sample s{cls, p.get(), p.get(), 1};
  if (!s.start || !s.stop) return hipErrorOutOfMemory;
  hipError_t e = hipEventRecord(s.start, st);
  if (e != hipSuccess) return e;
  e = launch();
  if (e != hipSuccess) return e;
  e = hipEventRecord(s.stop, st);
  p.pending.push_back(s);
  return e;
}

// ---- side stream for the time-batched GEMMs ------------------------------------------------------
// The weight-gradient and dx GEMMs of a finished chunk do not feed the sequential chain, so they
// run on a second stream (default priority) while the main stream carries on with the next
// steps.  Fork/join is by events only, so a caller may capture the whole run in a HIP graph.
struct SideStream {
  hipStream_t stream = nullptr;
  hipEvent_t full[2] = {nullptr, nullptr};   // main -> side: chunk buffer is complete
  hipEvent_t done[2] = {nullptr, nullptr};   // side -> main: chunk buffer may be overwritten
};
SideStream g_side[16];
std::mutex g_run_mutex;

hipError_t get_side_stream(SideStream** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= 16) return hipErrorInvalidDevice;
  SideStream& s = g_side[dev];
  if (!s.stream) {
    e = hipStreamCreateWithFlags(&s.stream, hipStreamNonBlocking);
    if (e != hipSuccess) return e;
    for (int i = 0; i < 2; ++i) {
      e = hipEventCreateWithFlags(&s.full[i], hipEventDisableTiming);
      if (e != hipSuccess) return e;
      e = hipEventCreateWithFlags(&s.done[i], hipEventDisableTiming);
      if (e != hipSuccess) return e;
    }
  }
  *out = &s;
  return hipSuccess;
}

#define HIP_TRY(expr)                                                                                 \
  do {                                                                                                \
    hipError_t e_ = (expr);                                                                           \
    if (e_ != hipSuccess) return set_error(MEBPTT_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

}  // namespace

extern "C" {

int mebptt_profile_enable(int32_t every_n) {
  if (every_n < 0) return set_error(MEBPTT_EINVAL, "every_n must be >= 0");
  g_prof.every_n = every_n;
  return MEBPTT_OK;
}

int mebptt_profile_collect(mebptt_profile* out) {
  if (!out) return set_error(MEBPTT_EINVAL, "out is NULL");
  std::memset(out, 0, sizeof *out);
  Profiler& p = g_prof;
  for (int c = 0; c < MEBPTT_K_CLASSES; ++c) {
    out->launches[c] = p.launches[c];
    p.launches[c] = 0;
  }
  int rc = MEBPTT_OK;
  for (Sample& s : p.runs) {
    float ms = 0.0f;
    hipError_t e = hipEventSynchronize(s.stop);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, s.start, s.stop);
    if (e != hipSuccess) {
      rc = set_error(MEBPTT_EHIP, "event timing failed: %s", hipGetErrorString(e));
    } else {
      out->forward_run_launches += s.launches;
      out->forward_run_ms += ms;
    }
    p.pool.push_back(s.start);
    p.pool.push_back(s.stop);
  }
  p.runs.clear();
  for (Sample& s : p.pending) {
    float ms = 0.0f;
    hipError_t e = hipEventSynchronize(s.stop);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, s.start, s.stop);
    if (e != hipSuccess) {
      rc = set_error(MEBPTT_EHIP, "event timing failed: %s", hipGetErrorString(e));
    } else {
      out->sampled[s.cls] += 1;
      out->sampled_ms[s.cls] += ms;
    }
    p.pool.push_back(s.start);
    p.pool.push_back(s.stop);
  }
  p.pending.clear();
  return rc;
}

size_t mebptt_unit_bytes(const mebptt_lstm_desc* desc) {
  if (!desc || desc->B < 1 || desc->H < 1) return 0;
  return make_dims(desc->B, 1, desc->H, desc->gemm_dtype ? 1 : 0, 0).unit * sizeof(float);
}

size_t mebptt_slot_pool_bytes(const mebptt_lstm_desc* desc, const mebptt_plan_t* plan) {
  if (!desc || !plan) return 0;
  size_t per = mebptt_unit_bytes(desc) * (plan->kind == MEBPTT_ISM ? 4 : 1);
  return align_up(per * (size_t)plan->m);
}

size_t mebptt_workspace_bytes(const mebptt_lstm_desc* desc) {
  if (check_desc(desc) != MEBPTT_OK) return 0;
  return layout(make_dims(desc->B, desc->I, desc->H, desc->gemm_dtype, desc->cell)).total;
}

int32_t mebptt_units_for_bytes(const mebptt_lstm_desc* desc, int32_t kind, size_t budget_bytes) {
  size_t per = mebptt_unit_bytes(desc) * (kind == MEBPTT_ISM ? 4 : 1);
  if (per == 0) return 0;
  size_t n = budget_bytes / per;
  return n > 0x7fffffff ? 0x7fffffff : (int32_t)n;
}

int mebptt_run(const mebptt_lstm_desc* desc, const mebptt_plan_t* plan, const float* W_ih, const float* W_hh,
               const float* b, const float* x, const float* dy, const float* h0, const float* c0, void* slots,
               size_t slots_bytes, void* workspace, size_t workspace_bytes, float* dW_ih, float* dW_hh, float* db,
               float* dh0, float* dc0, float* dx, float* y_out, mebptt_stats* stats, void* stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (!plan) return set_error(MEBPTT_EINVAL, "plan is NULL");
  if (plan->t != desc->t) return set_error(MEBPTT_ESHAPE, "plan is for t=%d, descriptor says t=%d", plan->t, desc->t);
  if (plan->ops.empty()) return set_error(MEBPTT_EINVAL, "plan carries no LSTM schedule (tables only)");
  if (!W_ih || !W_hh || !x || !dW_ih || !dW_hh || !db || !dh0 || !dc0)
    return set_error(MEBPTT_EINVAL, "a required device pointer is NULL");
  if (desc->loss == 0 && !dy) return set_error(MEBPTT_EINVAL, "dy is NULL but loss == 0");
  if (!slots) return set_error(MEBPTT_ENOMEM_SLOTS, "slots is NULL");
  if (!workspace) return set_error(MEBPTT_EWORKSPACE, "workspace is NULL");
  if (slots_bytes < mebptt_slot_pool_bytes(desc, plan))
    return set_error(MEBPTT_ENOMEM_SLOTS, "slot pool has %zu bytes, the plan needs %zu", slots_bytes,
                     mebptt_slot_pool_bytes(desc, plan));
  const Dims d = make_dims(desc->B, desc->I, desc->H, desc->gemm_dtype, desc->cell);
  const Workspace w = layout(d);
  if (workspace_bytes < w.total)
    return set_error(MEBPTT_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, w.total);
  if (misaligned(slots, ALIGN) || misaligned(workspace, ALIGN))
    return set_error(MEBPTT_EWORKSPACE, "slots and workspace must be 256-byte aligned");
  const void* f32ptrs[] = {W_ih, W_hh, b, x, dy, h0, c0, dW_ih, dW_hh, db, dh0, dc0, dx, y_out};
  for (const void* p : f32ptrs)
    if (p && misaligned(p, 16)) return set_error(MEBPTT_EINVAL, "device arrays must be 16-byte aligned");

  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  char* ws = reinterpret_cast<char*>(workspace);
  const size_t plane = (size_t)d.B * d.H;
  const size_t unit = d.unit;   // floats
  float* state = reinterpret_cast<float*>(ws + w.state);
  float* slot0 = reinterpret_cast<float*>(slots);
  int core_flip = 0;   // which of the two working-core buffers MEBPTT_LOC_CORE currently names
  auto loc = [&](int32_t l) -> float* {
    if (l >= 0) return slot0 + (size_t)l * unit;
    switch (l) {
      case MEBPTT_LOC_T0: return state;
      case MEBPTT_LOC_T1: return state + unit;
      case MEBPTT_LOC_CORE: return state + (core_flip ? 6 : 2) * unit;
      case MEBPTT_LOC_INIT: return state + 5 * unit;
      default: return nullptr;
    }
  };
  const int64_t pool_units = (int64_t)plan->m * (plan->kind == MEBPTT_ISM ? 4 : 1);
  // Host-side check of every location before anything is enqueued.
  for (const mebptt_op& op : plan->ops) {
    const int32_t locs[3] = {op.src, op.dst, op.prev};
    for (int i = 0; i < 3; ++i) {
      int32_t l = locs[i];
      if (i == 2 && l == MEBPTT_LOC_NONE) continue;
      int64_t span = (i == 1 && (op.keep || op.op == MEBPTT_OP_BWD)) ? 3 : 1;
      if (l >= 0 ? (l + span > pool_units) : (loc(l) == nullptr))
        return set_error(MEBPTT_EINVAL, "schedule names a location outside the pool");
    }
    if (op.step < 1 || op.step + op.count - 1 > desc->t) return set_error(MEBPTT_EINVAL, "schedule step out of range");
  }

  float* bp = reinterpret_cast<float*>(ws + w.bp);
  float* dc = reinterpret_cast<float*>(ws + w.dc);
  void* Wp = ws + w.Wp;
  void* WTh = ws + w.WTh;
  void* WTx = ws + w.WTx;
  const size_t op_b = d.op_bytes();

  // Set-up: operand copies of the weights, zeroed staging (the padding must stay zero), start state.
  HIP_TRY(timed(MEBPTT_K_SETUP, st, [&] { return launch_prep_weights(d, W_ih, W_hh, b, Wp, bp, WTh, WTx, st); }));
  HIP_TRY(timed(MEBPTT_K_SETUP, st, [&] { return launch_fill_zero(ws + w.dc, w.total - w.dc, st); }));
  HIP_TRY(timed(MEBPTT_K_SETUP, st, [&] {
    return launch_init_state(d, h0, c0, plan->kind == MEBPTT_ISM ? loc(MEBPTT_LOC_INIT) : loc(0), st);
  }));

  std::lock_guard<std::mutex> lock(g_run_mutex);   // the side stream and its events are shared
  SideStream* side = nullptr;
  HIP_TRY(get_side_stream(&side));
  hipStream_t st2 = side->stream;
  bool pending[2] = {false, false};   // side-stream work on chunk buffer i not yet joined
  int cur_chunk = -1;

  int64_t fwd = 0, bwd = 0;
  bool first_chunk = true;
  const int t = desc->t, CH = d.CH;
  const size_t dG_step = (size_t)d.BP * d.G4 * op_b;   // bytes of one step inside a dG chunk buffer
  const bool fuse = can_fuse_pair(d);

  // A backward step is held back until the next schedule entry is known: if that is a forward run
  // whose first step overwrites nothing the backward step reads, both go out in one launch.
  bool have_pending = false;
  BackwardArgs pend{};
  int pend_step = 0;

  // Launches the held-back backward step, alone or fused with one forward operation, then the
  // time-batched work of its chunk if the step completed one.
  auto flush_backward = [&](const float* x_s, const float* f_src, float* f_dst, float* f_gates) -> int {
    if (x_s) {
      HIP_TRY(timed(MEBPTT_K_PAIR, st, [&] {
        return launch_backward_forward_pair(d, pend, Wp, bp, x_s, f_src, f_dst, f_gates, st);
      }));
      ++fwd;
    } else {
      HIP_TRY(timed(MEBPTT_K_BACKWARD, st, [&] { return launch_backward(d, pend, st); }));
    }
    ++bwd;
    have_pending = false;
    const int s = pend_step;
    const int chunk = (s - 1) / CH, slot = (s - 1) % CH, buf = chunk & 1;
    if (slot == 0) {   // the chunk is complete: time-batched weight gradient and dx on the side stream
      const int nslots = (t - chunk * CH) < CH ? (t - chunk * CH) : CH;
      const size_t x_off = (size_t)chunk * CH * d.B * d.I;
      HIP_TRY(hipEventRecord(side->full[buf], st));
      HIP_TRY(hipStreamWaitEvent(st2, side->full[buf], 0));
      HIP_TRY(timed(MEBPTT_K_WGRAD, st2, [&] {
        hipError_t e = launch_transpose_x(d, x + x_off, nslots, ws + w.aT[buf], st2);
        if (e != hipSuccess) return e;
        return launch_wgrad(d, ws + w.dGT[buf], ws + w.aT[buf], nslots, first_chunk ? 0 : 1,
                            reinterpret_cast<float*>(ws + w.dWacc), st2);
      }));
      if (dx)
        HIP_TRY(timed(MEBPTT_K_DGRAD, st2, [&] {
          return launch_dgrad_gemm(d, WTx, d.I, ws + w.dG[buf], nslots, dx + x_off, d.I, st2);
        }));
      HIP_TRY(hipEventRecord(side->done[buf], st2));
      pending[buf] = true;
      first_chunk = false;
    }
    return MEBPTT_OK;
  };

  for (const mebptt_op& op : plan->ops) {
    if (op.op == MEBPTT_OP_FWD_RUN) {
      if (op.dst == MEBPTT_LOC_CORE) core_flip ^= 1;   // fresh core buffer: the held-back step may still read the other
      const float* cur = loc(op.src);
      // Measurement hook: one event pair around the back-to-back launches of a long run (all but
      // its first step, which may share a launch with a backward step).
      const bool bracket = g_prof.every_n > 0 && op.count >= 9 && g_prof.runs.size() < 100000;
      Sample run_sample{MEBPTT_K_FORWARD, nullptr, nullptr, op.count - 1};
      for (int j = 1; j <= op.count; ++j) {
        if (bracket && j == 2) {
          run_sample.start = g_prof.get();
          run_sample.stop = g_prof.get();
          if (!run_sample.start || !run_sample.stop) return set_error(MEBPTT_EHIP, "event creation failed");
          HIP_TRY(hipEventRecord(run_sample.start, st));
          g_prof.in_run = true;
        }
        const int step = op.step + j - 1;
        float* dst = (j == op.count) ? loc(op.dst)
                                     : (j == op.count - 1 ? loc(op.prev) : loc((j & 1) ? MEBPTT_LOC_T1 : MEBPTT_LOC_T0));
        float* gates = (j == op.count && op.keep) ? dst + unit : nullptr;
        const float* x_s = x + (size_t)(step - 1) * d.B * d.I;
        if (have_pending) {
          // units written by this forward step vs units read by the held-back backward step
          const float* w_lo = dst;
          const float* w_hi = dst + (gates ? 3 : 1) * unit;
          const bool clash = (w_lo < pend.state + 3 * unit && pend.state < w_hi) ||
                             (w_lo < pend.prev + unit && pend.prev < w_hi);
          if (fuse && !clash) {
            rc = flush_backward(x_s, cur, dst, gates);
            if (rc) return rc;
            cur = dst;
            continue;
          }
          rc = flush_backward(nullptr, nullptr, nullptr, nullptr);
          if (rc) return rc;
        }
        HIP_TRY(timed(MEBPTT_K_FORWARD, st, [&] { return launch_forward(d, Wp, bp, x_s, cur, dst, gates, st); }));
        cur = dst;
        ++fwd;
      }
      if (bracket) {
        g_prof.in_run = false;
        HIP_TRY(hipEventRecord(run_sample.stop, st));
        g_prof.runs.push_back(run_sample);
      }
    } else if (op.op == MEBPTT_OP_BWD) {
      if (have_pending) {
        rc = flush_backward(nullptr, nullptr, nullptr, nullptr);
        if (rc) return rc;
      }
      const int s = op.step;
      const int chunk = (s - 1) / CH, slot = (s - 1) % CH, buf = chunk & 1;
      if (chunk != cur_chunk) {   // first write into this chunk buffer: its previous user must be done
        if (pending[buf]) {
          HIP_TRY(hipStreamWaitEvent(st, side->done[buf], 0));
          pending[buf] = false;
        }
        cur_chunk = chunk;
      }
      pend = BackwardArgs{};
      pend.WTh = WTh;
      pend.dG_next = (s == t) ? nullptr : ws + w.dG[(s / CH) & 1] + (size_t)(s % CH) * dG_step;
      pend.state = loc(op.dst);
      pend.prev = loc(op.src);
      pend.dy_s = (desc->loss == 0 && s >= desc->dy_first_step) ? dy + (size_t)(s - desc->dy_first_step) * plane : nullptr;
      pend.dy_is_h = desc->loss == 1;
      pend.dc = dc;
      pend.dG_cur = ws + w.dG[buf] + (size_t)slot * dG_step;
      pend.dGT = ws + w.dGT[buf];
      pend.aT = ws + w.aT[buf];
      pend.col0 = slot * d.B;
      pend.y_out_s = y_out ? y_out + (size_t)(s - 1) * plane : nullptr;
      pend_step = s;
      have_pending = true;
    } else {
      return set_error(MEBPTT_EINVAL, "unknown schedule entry %d", op.op);
    }
  }
  if (have_pending) {
    rc = flush_backward(nullptr, nullptr, nullptr, nullptr);
    if (rc) return rc;
  }
  // LSTM: dh_0 = dG_1 W_hh ; dc_0 is the running cell gradient after step 1.
  // GRU:  dh_0 = dG_1 W_hh + dh_1 * z_1 (the running plane) ; there is no cell state: dc_0 = 0.
  HIP_TRY(timed(MEBPTT_K_DGRAD, st, [&] { return launch_dgrad_gemm(d, WTh, d.H, ws + w.dG[0], 1, dh0, d.H, st); }));
  if (d.cell == MEBPTT_CELL_LSTM) {
    HIP_TRY(timed(MEBPTT_K_SETUP, st, [&] { return launch_copy_plane(d, dc, dc0, 0, st); }));
  } else {
    HIP_TRY(timed(MEBPTT_K_SETUP, st, [&] { return launch_copy_plane(d, dc, dh0, 1, st); }));
    HIP_TRY(launch_copy_plane(d, dc, dc0, 2, st));
  }
  for (int i = 0; i < 2; ++i)   // join: everything is ordered before whatever follows on `st`
    if (pending[i]) HIP_TRY(hipStreamWaitEvent(st, side->done[i], 0));
  HIP_TRY(timed(MEBPTT_K_WGRAD, st, [&] {
    return launch_wgrad_finish(d, reinterpret_cast<const float*>(ws + w.dWacc), dW_ih, dW_hh, db, st);
  }));

  if (stats) {
    stats->forward_ops = fwd;
    stats->backward_ops = bwd;
    stats->peak = plan->peak;
    stats->reserved = 0;
    stats->peak_slot_bytes = (size_t)plan->peak * mebptt_unit_bytes(desc) * (plan->kind == MEBPTT_ISM ? 4 : 1);
  }
  return MEBPTT_OK;
}

}  // extern "C"
