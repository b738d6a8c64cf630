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

#include <algorithm>
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
  size_t Wp, bp, WTh, WTx, state, dWacc, dc, sync, dG[2], dGT[2], aT[2], ring, stage, total;
  size_t total_no_stage;   // what a run that issues no batched recomputation needs (the no-allocation path)
  int stage_steps;         // internal states the stage holds
};

// Internal states the recomputation stage holds: as many steps as a sweep launch carries, within
// 48 MiB; none where no backward-only sweep launch could consume them, and none on shapes that have
// the sweep launch with forward operations, which is the faster way there (H = 512, B = 256: 171 ms
// against 189 ms per gradient step).
constexpr size_t STAGE_MAX_BYTES = (size_t)48 << 20;
int recompute_stage_steps(const Dims& d) {
  if (!can_run_forward_batch(d) || !can_run_backward_sweep(d) || can_run_sweep(d)) return 0;
  const size_t state_bytes = 3 * d.unit * sizeof(float);
  const int n = (int)std::min<size_t>(STAGE_MAX_BYTES / state_bytes, (size_t)std::min(sweep_max_steps(), forward_batch_max_steps()));
  return n >= 4 ? n : 0;
}

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
  w.sync = take(forward_chain_sync_bytes());   // counters and status word of the resident launches: cleared with dc
  for (int i = 0; i < 2; ++i) w.dG[i] = take((size_t)d.CH * d.BP * d.G4 * op);
  for (int i = 0; i < 2; ++i) w.dGT[i] = take((size_t)d.G4 * d.KC * op);
  for (int i = 0; i < 2; ++i) w.aT[i] = take((size_t)d.NA * d.KC * op);
  w.ring = take(can_run_forward_chain(d) ? forward_chain_ring_bytes(d) : 0);
  w.total_no_stage = off;
  w.stage_steps = recompute_stage_steps(d);
  w.stage = take((size_t)w.stage_steps * 3 * unit);   // last: nothing ever clears it
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
  // A bracket that is still open: launches of one class on one stream share an event pair, up to
  // group_size(cls) of them, so that what the events themselves cost is spread over the group.
  struct Open {
    int cls = -1;
    hipStream_t st = nullptr;
    hipEvent_t start = nullptr;
    int64_t n = 0;
  } open;
  int64_t launches[MEBPTT_K_CLASSES] = {};
  int64_t sweep_forward_steps = 0;   // forward operations carried by sweep launches
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

// Launches of the sequential chain are bracketed in groups of up to eight consecutive launches of
// one class (an event pair around a single short launch adds microseconds to it); the batched GEMMs
// and the set-up kernels, which are long and not consecutive, one by one.
inline int group_size(int cls) {
  return (cls == MEBPTT_K_FORWARD || cls == MEBPTT_K_BACKWARD || cls == MEBPTT_K_PAIR) ? 8 : 1;
}

// Ends the open bracket, if any: its stop event goes onto its stream now.  Called before anything
// that is not a launch of the open class is put on that stream.
hipError_t close_group() {
  Profiler& p = g_prof;
  if (p.open.cls < 0) return hipSuccess;
  Sample s{p.open.cls, p.open.start, p.get(), p.open.n};
  p.open.cls = -1;
  if (!s.stop) {
    p.pool.push_back(s.start);
    return hipErrorOutOfMemory;
  }
  hipError_t e = hipEventRecord(s.stop, p.open.st);
  p.pending.push_back(s);
  return e;
}

// Brackets a group of launches with events when its first launch falls on the sampling grid.
template <class F>
hipError_t timed(int cls, hipStream_t st, F&& launch) {
  Profiler& p = g_prof;
  if (p.every_n <= 0) return launch();
  if (p.open.cls >= 0 && (p.open.cls != cls || p.open.st != st || p.in_run)) {
    hipError_t e = close_group();
    if (e != hipSuccess) return e;
  }
  const int64_t index = p.launches[cls]++;
  if (p.open.cls < 0) {
    const bool sample = (index % p.every_n) == 0 && p.pending.size() < 200000 && !p.in_run;
    if (!sample) return launch();
    hipEvent_t start = p.get();
    if (!start) return hipErrorOutOfMemory;
    hipError_t e = hipEventRecord(start, st);
    if (e != hipSuccess) {
      p.pool.push_back(start);
      return e;
    }
    p.open.cls = cls;
    p.open.st = st;
    p.open.start = start;
    p.open.n = 0;
  }
  hipError_t e = launch();
  if (e != hipSuccess) return e;
  if (++p.open.n >= group_size(cls)) e = close_group();
  return e;
}

// ---- side stream for the time-batched GEMMs ------------------------------------------------------
// The weight-gradient and dx GEMMs of a finished chunk do not feed the sequential chain, so they
// run on a second stream (default priority) while the main stream carries on with the next
// steps.  Fork/join is by events only, so a caller may capture the whole run in a HIP graph.
// One such stream and four events exist per device, created by the first mebptt_run on that
// device and destroyed by mebptt_shutdown; g_run_mutex serialises the enqueue of runs because
// they share them.
constexpr int MAX_DEVICES = 16;
struct SideStream {
  hipStream_t stream = nullptr;
  hipEvent_t full[2] = {nullptr, nullptr};   // main -> side: chunk buffer is complete
  hipEvent_t done[2] = {nullptr, nullptr};   // side -> main: chunk buffer may be overwritten
};
SideStream g_side[MAX_DEVICES];
std::mutex g_run_mutex;
// Forward-chain launches want every compute unit of the device; two of them from different streams
// would each hold a part of the chip and wait for the rest.  The last run that used them records
// this event when its work is enqueued and the next such run makes its stream wait for it.
bool g_chain_enabled = true;

// The resident launches (forward chains, sweeps) are laid out for a device of 8 XCDs with 32 compute
// units each; on anything else (a partitioned device, masked compute units) they would only raise
// their status word, so there the launch-per-step path is used from the start.  Cached per device;
// called with g_run_mutex held.
int g_device_cus[16] = {};   // 0: not asked yet
bool device_fits_resident_launches() {
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 16) return false;
  if (g_device_cus[dev] == 0) {
    int n = 0;
    if (hipDeviceGetAttribute(&n, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess) n = -1;
    g_device_cus[dev] = n > 0 ? n : -1;
  }
  return g_device_cus[dev] == 256;
}
hipEvent_t g_chain_done[MAX_DEVICES] = {};
bool g_chain_recorded[MAX_DEVICES] = {};

hipError_t get_side_stream(SideStream** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
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

// ---- workspaces that mebptt_prepare has filled ---------------------------------------------------
// Host-side record only (the device memory is the caller's): which workspace holds the operand
// copies of which weights for which shape, so that mebptt_run_prepared can refuse a workspace
// that was never prepared or was prepared for another shape.
struct Prepared {
  const void* workspace;
  int B, I, H, dtype, cell;
};
std::vector<Prepared> g_prepared;
std::mutex g_prepared_mutex;

void remember_prepared(const void* ws, const Dims& d) {
  std::lock_guard<std::mutex> lock(g_prepared_mutex);
  for (Prepared& p : g_prepared)
    if (p.workspace == ws) {
      p = Prepared{ws, d.B, d.I, d.H, d.dtype, d.cell};
      return;
    }
  if (g_prepared.size() >= 64) g_prepared.erase(g_prepared.begin());   // oldest record goes
  g_prepared.push_back(Prepared{ws, d.B, d.I, d.H, d.dtype, d.cell});
}

bool is_prepared(const void* ws, const Dims& d) {
  std::lock_guard<std::mutex> lock(g_prepared_mutex);
  for (const Prepared& p : g_prepared)
    if (p.workspace == ws) return p.B == d.B && p.I == d.I && p.H == d.H && p.dtype == d.dtype && p.cell == d.cell;
  return false;
}

// ---- static scratch for callers that cannot allocate ---------------------------------------------
// mebptt_run_static keeps its workspace here instead of taking one from the caller.  In host code
// the array's name is only a handle: its device address is looked up once per device with
// hipGetSymbolAddress and that pointer is what kernels receive.
static __device__ __align__(256) unsigned char scratch[MEBPTT_STATIC_WORKSPACE_BYTES];
void* g_scratch_ptr[MAX_DEVICES] = {};
std::mutex g_scratch_mutex;

hipError_t get_scratch(void** out) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= MAX_DEVICES) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_scratch_mutex);
  if (!g_scratch_ptr[dev]) {
    void* ptr = nullptr;
    e = hipGetSymbolAddress(&ptr, HIP_SYMBOL(scratch));
    if (e != hipSuccess) return e;
    if (!ptr) return hipErrorInvalidSymbol;
    g_scratch_ptr[dev] = ptr;
  }
  *out = g_scratch_ptr[dev];
  return hipSuccess;
}

__global__ void null_kernel() {}

#define HIP_TRY(expr)                                                                                 \
  do {                                                                                                \
    hipError_t e_ = (expr);                                                                           \
    if (e_ != hipSuccess) return set_error(MEBPTT_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

enum RunMode {
  RUN_FULL,       // operand copies of the weights are built inside the call
  RUN_PREPARED,   // mebptt_prepare has built them in this workspace
  RUN_STATIC      // as RUN_FULL, on one stream, with nothing created or allocated
};

int run_impl(RunMode mode, const mebptt_lstm_desc* desc, const mebptt_plan_t* plan, const float* W_ih,
             const float* W_hh, const float* b, const float* x, const float* dy, const float* h0, const float* c0,
             void* slots, size_t slots_bytes, void* workspace, size_t workspace_bytes, float* dW_ih, float* dW_hh,
             float* db, float* dh0, float* dc0, float* dx, float* y_out, mebptt_stats* stats, void* stream);

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
  if (close_group() != hipSuccess) return set_error(MEBPTT_EHIP, "closing an event bracket failed");
  for (int c = 0; c < MEBPTT_K_CLASSES; ++c) {
    out->launches[c] = p.launches[c];
    p.launches[c] = 0;
  }
  out->sweep_forward_steps = p.sweep_forward_steps;
  p.sweep_forward_steps = 0;
  int rc = MEBPTT_OK;
  for (Sample& s : p.runs) {
    float ms = 0.0f;
    hipError_t e = hipEventSynchronize(s.stop);
    if (e == hipSuccess) e = hipEventElapsedTime(&ms, s.start, s.stop);
    if (e != hipSuccess) {
      rc = set_error(MEBPTT_EHIP, "event timing failed: %s", hipGetErrorString(e));
    } else if (s.cls == MEBPTT_K_CHAIN) {
      out->chain_steps += s.launches;
      out->chain_ms += ms;
    } else if (s.cls == MEBPTT_K_SWEEP) {
      out->sweep_steps += s.launches;
      out->sweep_ms += ms;
    } else if (s.cls == MEBPTT_K_FWD_BATCH) {
      out->batch_steps += s.launches;
      out->batch_ms += ms;
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
      out->sampled[s.cls] += s.launches;
      out->sampled_groups[s.cls] += 1;
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
  return run_impl(RUN_FULL, desc, plan, W_ih, W_hh, b, x, dy, h0, c0, slots, slots_bytes, workspace, workspace_bytes,
                  dW_ih, dW_hh, db, dh0, dc0, dx, y_out, stats, stream);
}

int mebptt_prepare(const mebptt_lstm_desc* desc, const float* W_ih, const float* W_hh, const float* b, void* workspace,
                   size_t workspace_bytes, void* stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (!W_ih || !W_hh) return set_error(MEBPTT_EINVAL, "a required device pointer is NULL");
  if (!workspace) return set_error(MEBPTT_EWORKSPACE, "workspace is NULL");
  const Dims d = make_dims(desc->B, desc->I, desc->H, desc->gemm_dtype, desc->cell);
  const Workspace w = layout(d);
  if (workspace_bytes < w.total)
    return set_error(MEBPTT_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, w.total);
  if (misaligned(workspace, ALIGN)) return set_error(MEBPTT_EWORKSPACE, "workspace must be 256-byte aligned");
  if (misaligned(W_ih, 16) || misaligned(W_hh, 16) || (b && misaligned(b, 16)))
    return set_error(MEBPTT_EINVAL, "device arrays must be 16-byte aligned");
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  char* ws = reinterpret_cast<char*>(workspace);
  std::lock_guard<std::mutex> lock(g_run_mutex);   // the measurement hooks' state is shared with runs
  HIP_TRY(timed(MEBPTT_K_SETUP, st, [&] {
    return launch_prep_weights(d, W_ih, W_hh, b, ws + w.Wp, reinterpret_cast<float*>(ws + w.bp), ws + w.WTh, ws + w.WTx, st);
  }));
  HIP_TRY(timed(MEBPTT_K_SETUP, st, [&] { return launch_fill_zero(ws + w.dc, w.total_no_stage - w.dc, st); }));
  remember_prepared(workspace, d);
  return MEBPTT_OK;
}

int mebptt_run_prepared(const mebptt_lstm_desc* desc, const mebptt_plan_t* plan, const float* x, const float* dy,
                        const float* h0, const float* c0, void* slots, size_t slots_bytes, void* workspace,
                        size_t workspace_bytes, float* dW_ih, float* dW_hh, float* db, float* dh0, float* dc0, float* dx,
                        float* y_out, mebptt_stats* stats, void* stream) {
  return run_impl(RUN_PREPARED, desc, plan, nullptr, nullptr, nullptr, x, dy, h0, c0, slots, slots_bytes, workspace,
                  workspace_bytes, dW_ih, dW_hh, db, dh0, dc0, dx, y_out, stats, stream);
}

int mebptt_run_status(const mebptt_lstm_desc* desc, const void* workspace, size_t workspace_bytes, void* stream,
                      int32_t* status) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (!status) return set_error(MEBPTT_EINVAL, "status is NULL");
  if (!workspace) return set_error(MEBPTT_EWORKSPACE, "workspace is NULL");
  const Workspace w = layout(make_dims(desc->B, desc->I, desc->H, desc->gemm_dtype, desc->cell));
  if (workspace_bytes < w.total)
    return set_error(MEBPTT_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, w.total);
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  HIP_TRY(hipStreamSynchronize(st));
  unsigned word = 0;
  HIP_TRY(hipMemcpy(&word, reinterpret_cast<const char*>(workspace) + w.sync + forward_chain_status_offset(), sizeof word,
                    hipMemcpyDeviceToHost));
  *status = (int32_t)word;
  return MEBPTT_OK;
}

int mebptt_resident_wait_limit(int64_t ticks) {
  std::lock_guard<std::mutex> lock(g_run_mutex);
  set_resident_wait_ticks((long long)ticks);
  return MEBPTT_OK;
}

int mebptt_forward_chain_enable(int32_t on) {
  std::lock_guard<std::mutex> lock(g_run_mutex);
  g_chain_enabled = on != 0;
  return MEBPTT_OK;
}

int mebptt_shutdown(void) {
  std::lock_guard<std::mutex> lock(g_run_mutex);
  int rc = MEBPTT_OK;
  auto drop = [&](hipError_t e) {
    if (e != hipSuccess) rc = set_error(MEBPTT_EHIP, "releasing a library resource failed: %s", hipGetErrorString(e));
  };
  int cur = 0;
  const bool have_dev = hipGetDevice(&cur) == hipSuccess;
  for (int dev = 0; dev < MAX_DEVICES; ++dev) {
    SideStream& s = g_side[dev];
    if (!s.stream) continue;
    drop(hipSetDevice(dev));
    drop(hipStreamSynchronize(s.stream));
    for (int i = 0; i < 2; ++i) {
      if (s.full[i]) drop(hipEventDestroy(s.full[i]));
      if (s.done[i]) drop(hipEventDestroy(s.done[i]));
    }
    drop(hipStreamDestroy(s.stream));
    s = SideStream{};
  }
  for (int dev = 0; dev < MAX_DEVICES; ++dev) {
    if (g_chain_done[dev]) drop(hipEventDestroy(g_chain_done[dev]));
    g_chain_done[dev] = nullptr;
    g_chain_recorded[dev] = false;
  }
  if (have_dev) drop(hipSetDevice(cur));
  Profiler& p = g_prof;
  for (Sample& sm : p.pending) {
    p.pool.push_back(sm.start);
    p.pool.push_back(sm.stop);
  }
  for (Sample& sm : p.runs) {
    p.pool.push_back(sm.start);
    p.pool.push_back(sm.stop);
  }
  p.pending.clear();
  p.runs.clear();
  for (hipEvent_t e : p.pool)
    if (e) drop(hipEventDestroy(e));
  p.pool.clear();
  p.every_n = 0;
  {
    std::lock_guard<std::mutex> lk(g_prepared_mutex);
    g_prepared.clear();
  }
  return rc;
}

int mebptt_null_launch_us(int32_t launches, void* stream, double* out_us) {
  if (launches < 1 || launches > 100000) return set_error(MEBPTT_EINVAL, "launches must be in [1, 100000]");
  if (!out_us) return set_error(MEBPTT_EINVAL, "out_us is NULL");
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  hipEvent_t a = nullptr, z = nullptr;
  HIP_TRY(hipEventCreate(&a));
  hipError_t e = hipEventCreate(&z);
  if (e == hipSuccess) {
    for (int i = 0; i < 16; ++i) null_kernel<<<dim3(256), dim3(256), 0, st>>>();   // warm-up
    e = hipEventRecord(a, st);
  }
  if (e == hipSuccess) {
    for (int i = 0; i < launches; ++i) null_kernel<<<dim3(256), dim3(256), 0, st>>>();
    e = hipGetLastError();
  }
  if (e == hipSuccess) e = hipEventRecord(z, st);
  if (e == hipSuccess) e = hipEventSynchronize(z);
  float ms = 0.0f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, a, z);
  (void)hipEventDestroy(a);
  if (z) (void)hipEventDestroy(z);
  if (e != hipSuccess) return set_error(MEBPTT_EHIP, "null-launch timing failed: %s", hipGetErrorString(e));
  *out_us = (double)ms * 1e3 / launches;
  return MEBPTT_OK;
}

int32_t mebptt_chunk_steps(const mebptt_lstm_desc* desc) {
  int rc = check_desc(desc);
  if (rc) return rc;
  return make_dims(desc->B, desc->I, desc->H, desc->gemm_dtype, desc->cell).CH;
}

int32_t mebptt_stage_steps(const mebptt_lstm_desc* desc) {
  int rc = check_desc(desc);
  if (rc) return rc;
  return recompute_stage_steps(make_dims(desc->B, desc->I, desc->H, desc->gemm_dtype, desc->cell));
}

int mebptt_measure_gemms(const mebptt_lstm_desc* desc, void* workspace, size_t workspace_bytes, int32_t reps,
                         void* stream, double* wgrad_us, double* dgrad_us) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (reps < 1 || reps > 10000 || !wgrad_us || !dgrad_us) return set_error(MEBPTT_EINVAL, "reps must be in [1, 10000] and the outputs non-NULL");
  if (!workspace) return set_error(MEBPTT_EWORKSPACE, "workspace is NULL");
  const Dims d = make_dims(desc->B, desc->I, desc->H, desc->gemm_dtype, desc->cell);
  const Workspace w = layout(d);
  if (workspace_bytes < w.total)
    return set_error(MEBPTT_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, w.total);
  if (misaligned(workspace, ALIGN)) return set_error(MEBPTT_EWORKSPACE, "workspace must be 256-byte aligned");
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  char* ws = reinterpret_cast<char*>(workspace);
  std::lock_guard<std::mutex> lock(g_run_mutex);
  hipEvent_t ev[3] = {nullptr, nullptr, nullptr};
  for (hipEvent_t& e : ev) HIP_TRY(hipEventCreate(&e));
  // dx goes to the dG buffer the GEMM does not read (scratch of sufficient size: CH*B*I floats <= CH*BP*G4 operand bytes)
  float* dx_scratch = reinterpret_cast<float*>(ws + w.dG[1]);
  hipError_t e = hipSuccess;
  for (int pass = 0; pass < 2 && e == hipSuccess; ++pass) {   // first pass warms up
    e = hipEventRecord(ev[0], st);
    for (int i = 0; i < reps && e == hipSuccess; ++i)
      e = launch_wgrad(d, ws + w.dGT[0], ws + w.aT[0], d.CH, 1, reinterpret_cast<float*>(ws + w.dWacc), st);
    if (e == hipSuccess) e = hipEventRecord(ev[1], st);
    for (int i = 0; i < reps && e == hipSuccess; ++i)
      e = launch_dx_gemm(d, ws + w.WTx, ws + w.dG[0], d.CH, dx_scratch, ws + w.dGT[1], w.dGT[1] - w.dGT[0], st);
    if (e == hipSuccess) e = hipEventRecord(ev[2], st);
    if (e == hipSuccess) e = hipEventSynchronize(ev[2]);
  }
  float ms_w = 0.0f, ms_d = 0.0f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms_w, ev[0], ev[1]);
  if (e == hipSuccess) e = hipEventElapsedTime(&ms_d, ev[1], ev[2]);
  for (hipEvent_t& x : ev) (void)hipEventDestroy(x);
  if (e != hipSuccess) return set_error(MEBPTT_EHIP, "GEMM timing failed: %s", hipGetErrorString(e));
  *wgrad_us = (double)ms_w * 1e3 / reps;
  *dgrad_us = (double)ms_d * 1e3 / reps;
  return MEBPTT_OK;
}

int mebptt_measure_forward_stream(const mebptt_lstm_desc* desc, void* workspace, size_t workspace_bytes, int32_t reps,
                                  void* stream, double* us_per_launch, double* delivered_bytes) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (reps < 1 || reps > 10000 || !us_per_launch || !delivered_bytes)
    return set_error(MEBPTT_EINVAL, "reps must be in [1, 10000] and the outputs non-NULL");
  if (!workspace) return set_error(MEBPTT_EWORKSPACE, "workspace is NULL");
  const Dims d = make_dims(desc->B, desc->I, desc->H, desc->gemm_dtype, desc->cell);
  const Workspace w = layout(d);
  if (workspace_bytes < w.total)
    return set_error(MEBPTT_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, w.total);
  if (misaligned(workspace, ALIGN)) return set_error(MEBPTT_EWORKSPACE, "workspace must be 256-byte aligned");
  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  char* ws = reinterpret_cast<char*>(workspace);
  std::lock_guard<std::mutex> lock(g_run_mutex);
  hipEvent_t ev[2] = {nullptr, nullptr};
  for (hipEvent_t& e : ev) HIP_TRY(hipEventCreate(&e));
  size_t delivered = 0;
  hipError_t e = hipSuccess;
  for (int pass = 0; pass < 2 && e == hipSuccess; ++pass) {   // first pass warms up
    e = hipEventRecord(ev[0], st);
    for (int i = 0; i < reps && e == hipSuccess; ++i)
      e = launch_forward_stream(d, ws + w.Wp, ws + w.state, w.dWacc - w.state, reinterpret_cast<float*>(ws + w.dc), &delivered, st);
    if (e == hipSuccess) e = hipEventRecord(ev[1], st);
    if (e == hipSuccess) e = hipEventSynchronize(ev[1]);
  }
  float ms = 0.0f;
  if (e == hipSuccess) e = hipEventElapsedTime(&ms, ev[0], ev[1]);
  for (hipEvent_t& x : ev) (void)hipEventDestroy(x);
  if (e != hipSuccess) return set_error(MEBPTT_EHIP, "streaming measurement failed: %s", hipGetErrorString(e));
  *us_per_launch = (double)ms * 1e3 / reps;
  *delivered_bytes = (double)delivered;
  return MEBPTT_OK;
}

size_t mebptt_static_workspace_bytes(void) { return MEBPTT_STATIC_WORKSPACE_BYTES; }

int mebptt_run_static(const mebptt_lstm_desc* desc, const mebptt_plan_t* plan, const float* W_ih, const float* W_hh,
                      const float* b, const float* x, const float* dy, const float* h0, const float* c0, void* slots,
                      size_t slots_bytes, float* dW_ih, float* dW_hh, float* db, float* dh0, float* dc0, float* dx,
                      float* y_out, mebptt_stats* stats, void* stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  const size_t need = layout(make_dims(desc->B, desc->I, desc->H, desc->gemm_dtype, desc->cell)).total_no_stage;
  if (need > MEBPTT_STATIC_WORKSPACE_BYTES)
    return set_error(MEBPTT_EWORKSPACE, "this shape needs %zu bytes of workspace; the static scratch holds %zu", need,
                     (size_t)MEBPTT_STATIC_WORKSPACE_BYTES);
  void* ptr = nullptr;
  HIP_TRY(get_scratch(&ptr));
  return run_impl(RUN_STATIC, desc, plan, W_ih, W_hh, b, x, dy, h0, c0, slots, slots_bytes, ptr,
                  MEBPTT_STATIC_WORKSPACE_BYTES, dW_ih, dW_hh, db, dh0, dc0, dx, y_out, stats, stream);
}

}  // extern "C"

namespace {

int run_impl(RunMode mode, const mebptt_lstm_desc* desc, const mebptt_plan_t* plan, const float* W_ih,
             const float* W_hh, const float* b, const float* x, const float* dy, const float* h0, const float* c0,
             void* slots, size_t slots_bytes, void* workspace, size_t workspace_bytes, float* dW_ih, float* dW_hh,
             float* db, float* dh0, float* dc0, float* dx, float* y_out, mebptt_stats* stats, void* stream) {
  int rc = check_desc(desc);
  if (rc) return rc;
  if (!plan) return set_error(MEBPTT_EINVAL, "plan is NULL");
  if (plan->t != desc->t) return set_error(MEBPTT_ESHAPE, "plan is for t=%d, descriptor says t=%d", plan->t, desc->t);
  if (plan->ops.empty()) return set_error(MEBPTT_EINVAL, "plan carries no LSTM schedule (tables only)");
  if (mode != RUN_PREPARED && (!W_ih || !W_hh)) return set_error(MEBPTT_EINVAL, "a required device pointer is NULL");
  if (!x || !dW_ih || !dW_hh || !db || !dh0 || !dc0) return set_error(MEBPTT_EINVAL, "a required device pointer is NULL");
  if (desc->loss == 0 && !dy) return set_error(MEBPTT_EINVAL, "dy is NULL but loss == 0");
  if (!slots) return set_error(MEBPTT_ENOMEM_SLOTS, "slots is NULL");
  if (!workspace) return set_error(MEBPTT_EWORKSPACE, "workspace is NULL");
  if (slots_bytes < mebptt_slot_pool_bytes(desc, plan))
    return set_error(MEBPTT_ENOMEM_SLOTS, "slot pool has %zu bytes, the plan needs %zu", slots_bytes,
                     mebptt_slot_pool_bytes(desc, plan));
  const Dims d = make_dims(desc->B, desc->I, desc->H, desc->gemm_dtype, desc->cell);
  const Workspace w = layout(d);
  const size_t ws_need = mode == RUN_STATIC ? w.total_no_stage : w.total;   // the no-allocation path never uses the stage
  if (workspace_bytes < ws_need)
    return set_error(MEBPTT_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes, ws_need);
  if (misaligned(slots, ALIGN) || misaligned(workspace, ALIGN))
    return set_error(MEBPTT_EWORKSPACE, "slots and workspace must be 256-byte aligned");
  const void* f32ptrs[] = {W_ih, W_hh, b, x, dy, h0, c0, dW_ih, dW_hh, db, dh0, dc0, dx, y_out};
  for (const void* p : f32ptrs)
    if (p && misaligned(p, 16)) return set_error(MEBPTT_EINVAL, "device arrays must be 16-byte aligned");
  if (mode == RUN_PREPARED && !is_prepared(workspace, d))
    return set_error(MEBPTT_EWORKSPACE, "workspace was not prepared for this shape: call mebptt_prepare first");

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
  const int units_per_budget = plan->kind == MEBPTT_ISM ? 4 : 1;
  const int64_t pool_units = (int64_t)plan->m * units_per_budget;
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
  // Slot units the launches of this run are handed, as the executor hands them out: the highest
  // unit index (+ span) among all state arguments.  This, not the planner's simulation, is what
  // the statistics report as the peak.
  int64_t high_water = 0;
  auto touch = [&](int32_t l, int span) {
    if (l >= 0) high_water = std::max<int64_t>(high_water, (int64_t)l + span);
  };

  float* bp = reinterpret_cast<float*>(ws + w.bp);
  float* dc = reinterpret_cast<float*>(ws + w.dc);
  void* Wp = ws + w.Wp;
  void* WTh = ws + w.WTh;
  void* WTx = ws + w.WTx;
  const size_t op_b = d.op_bytes();
  const int t = desc->t, CH = d.CH;
  const bool use_profiler = mode != RUN_STATIC;   // event brackets create events: not in the no-allocation path
  auto tm = [&](int cls, hipStream_t s, auto&& launch) -> hipError_t {
    return use_profiler ? timed(cls, s, launch) : launch();
  };
  // A launch that carries `carried` operations (forward chain, sweep, forward batch): the measurement
  // hook brackets each of them whole, on the run's stream, and records what it carried.
  auto whole_launch = [&](int cls, int carried, hipStream_t s, auto&& launch) -> int {
    const bool bracket = use_profiler && g_prof.every_n > 0 && g_prof.runs.size() < 100000;
    if (use_profiler) HIP_TRY(close_group());
    Sample smp{cls, nullptr, nullptr, carried};
    if (bracket) {
      smp.start = g_prof.get();
      smp.stop = g_prof.get();
      if (!smp.start || !smp.stop) return set_error(MEBPTT_EHIP, "event creation failed");
      HIP_TRY(hipEventRecord(smp.start, s));
    }
    HIP_TRY(launch());
    if (bracket) {
      HIP_TRY(hipEventRecord(smp.stop, s));
      g_prof.runs.push_back(smp);
    }
    if (use_profiler && g_prof.every_n > 0) ++g_prof.launches[cls];
    return MEBPTT_OK;
  };

  std::lock_guard<std::mutex> lock(g_run_mutex);   // side stream, events, profiler and static scratch are shared
  if (g_prof.open.cls >= 0) {   // a run that failed midway left its last bracket open: forget it
    g_prof.pool.push_back(g_prof.open.start);
    g_prof.open.cls = -1;
  }

  // Set-up: operand copies of the weights, zeroed staging (the padding must stay zero), start state.
  if (mode != RUN_PREPARED) {
    HIP_TRY(tm(MEBPTT_K_SETUP, st, [&] { return launch_prep_weights(d, W_ih, W_hh, b, Wp, bp, WTh, WTx, st); }));
    HIP_TRY(tm(MEBPTT_K_SETUP, st, [&] { return launch_fill_zero(ws + w.dc, w.total_no_stage - w.dc, st); }));
  } else {
    // The staging keeps what the previous run left.  Only the running gradient plane must start
    // at zero, and -- when the last chunk in time is short and its K is padded -- the operand
    // columns between its last step and the padded K, which a full chunk of the previous run
    // filled.
    HIP_TRY(tm(MEBPTT_K_SETUP, st, [&] { return launch_fill_zero(ws + w.dc, w.dG[0] - w.dc, st); }));
    const int last_chunk = (t - 1) / CH, nslots = t - last_chunk * CH;
    const int cols = nslots * d.B, kstep = d.dtype ? 32 : 16;
    if (cols % kstep != 0)
      HIP_TRY(tm(MEBPTT_K_SETUP, st, [&] {
        return launch_zero_operand_columns(d, ws + w.dGT[last_chunk & 1], ws + w.aT[last_chunk & 1], cols,
                                           round_up(cols, kstep), st);
      }));
  }
  HIP_TRY(tm(MEBPTT_K_SETUP, st, [&] {
    return launch_init_state(d, h0, c0, plan->kind == MEBPTT_ISM ? loc(MEBPTT_LOC_INIT) : loc(0), st);
  }));
  if (plan->kind != MEBPTT_ISM) touch(0, 1);

  // The time-batched GEMMs go to the side stream where the sequential work runs as resident
  // launches (they then fill the gaps those launches leave: measured 1 % faster on H = 1024).
  // Beside launch-per-step kernels, which fill the device on their own, the two only get in each
  // other's way (H = 2048: 2.8 % slower, H = 4096: 1.4 %), so there -- and in the no-allocation
  // path, which creates no stream and no event -- they stay on the caller's stream in the same order.
  const bool resident_ok = mode != RUN_STATIC && g_chain_enabled && device_fits_resident_launches();
  SideStream* side = nullptr;
  if (resident_ok && (can_run_forward_chain(d) || can_run_backward_sweep(d))) HIP_TRY(get_side_stream(&side));
  hipStream_t st2 = side ? side->stream : st;
  bool pending[2] = {false, false};   // side-stream work on chunk buffer i not yet joined
  int cur_chunk = -1;

  int64_t fwd = 0, bwd = 0;
  int64_t gemm_mark[2] = {INT64_MIN / 2, INT64_MIN / 2};   // fwd + bwd when the GEMMs reading chunk buffer i were issued
  bool first_chunk = true;
  const size_t dG_step = (size_t)d.BP * d.G4 * op_b;   // bytes of one step inside a dG chunk buffer
  const bool fuse = can_fuse_pair(d);

  // A backward step is held back until the next schedule entry is known: if that is a forward run
  // whose first step overwrites nothing the backward step reads, both go out in one launch.
  bool have_pending = false;
  BackwardArgs pend{};
  int pend_step = 0;
  int chain_order_dev = -1;   // device whose chain-ordering event this run waits for and records

  // The time-batched weight gradient and dx of a chunk whose first step has just been back-propagated.
  auto complete_chunk = [&](int chunk) -> int {
    const int buf = chunk & 1;
    const int nslots = (t - chunk * CH) < CH ? (t - chunk * CH) : CH;
    const size_t x_off = (size_t)chunk * CH * d.B * d.I;
    if (side) {
      HIP_TRY(hipEventRecord(side->full[buf], st));
      HIP_TRY(hipStreamWaitEvent(st2, side->full[buf], 0));
    }
    HIP_TRY(tm(MEBPTT_K_WGRAD, st2, [&] {
      hipError_t e = launch_transpose_x(d, x + x_off, nslots, ws + w.aT[buf], st2);
      if (e != hipSuccess) return e;
      return launch_wgrad(d, ws + w.dGT[buf], ws + w.aT[buf], nslots, first_chunk ? 0 : 1,
                          reinterpret_cast<float*>(ws + w.dWacc), st2);
    }));
    if (dx)
      HIP_TRY(tm(MEBPTT_K_DGRAD, st2, [&] {
        // the chunk's dG^T buffer is free from here (its dW GEMM is ahead on the same stream) until the
        // chunk after next fills it: the dx GEMM may keep partial sums there
        return launch_dx_gemm(d, WTx, ws + w.dG[buf], nslots, dx + x_off, ws + w.dGT[buf], w.dGT[1] - w.dGT[0], st2);
      }));
    if (side) {
      HIP_TRY(hipEventRecord(side->done[buf], st2));
      pending[buf] = true;
    }
    gemm_mark[buf] = fwd + bwd;
    first_chunk = false;
    return MEBPTT_OK;
  };
  // A sweep launch that starts in chunk c may run on into chunk c - 1, whose buffers the GEMMs of
  // chunk c + 1 read: it then waits for them.  Worth it only if they were issued long enough ago to
  // be done -- counted in operations enqueued on the run's stream since (a chunk's GEMMs take about
  // as long as 15 - 30 of them; thresholds of 8, 16, 32 and 64 were measured, 16 is the best on the
  // workloads cfg2 and cfg4).  Launches that follow each other directly therefore end at the chunk
  // boundary, as they always did; with the GEMMs on the run's own stream there is nothing to wait for.
  constexpr int64_t CROSS_MIN_OPS = 16;
  auto may_cross = [&](int chunk) { return !side || (fwd + bwd) - gemm_mark[(chunk - 1) & 1] >= CROSS_MIN_OPS; };
  // Before the first write into a chunk's buffers: their previous user (the GEMMs of the chunk
  // two before) must be done.
  auto begin_chunk = [&](int chunk) -> int {
    if (chunk != cur_chunk) {
      const int buf = chunk & 1;
      if (pending[buf]) {
        HIP_TRY(hipStreamWaitEvent(st, side->done[buf], 0));
        pending[buf] = false;
      }
      cur_chunk = chunk;
    }
    return MEBPTT_OK;
  };

  // Launches the held-back backward step, alone or fused with one forward operation, then the
  // time-batched work of its chunk if the step completed one.
  auto flush_backward = [&](const float* x_s, const float* f_src, float* f_dst, float* f_gates) -> int {
    if (x_s) {
      HIP_TRY(tm(MEBPTT_K_PAIR, st, [&] {
        return launch_backward_forward_pair(d, pend, Wp, bp, x_s, f_src, f_dst, f_gates, st);
      }));
      ++fwd;
    } else {
      HIP_TRY(tm(MEBPTT_K_BACKWARD, st, [&] { return launch_backward(d, pend, st); }));
    }
    ++bwd;
    have_pending = false;
    const int s = pend_step;
    if ((s - 1) % CH == 0) return complete_chunk((s - 1) / CH);   // the chunk is complete
    return MEBPTT_OK;
  };

  // Forward operations that follow each other (a forward run, or consecutive runs each starting
  // from the state the one before left) form a chain; on shapes whose weights fit on the chip a
  // chain goes out as forward-chain launches of up to forward_chain_max_steps() steps instead of
  // one launch per step.  Not in the no-allocation path, which owns no event to keep two such runs
  // from overlapping on the device.
  const bool chain_ok = resident_ok && can_run_forward_chain(d);
  constexpr int CHAIN_MIN_STEPS = 2;     // two steps in one launch already beat two launches (measured on the paper's 256-wide model)
  unsigned chain_base = 0;        // arrivals left in the group counters by this run's earlier chain launches
  unsigned chain_launches = 0;    // chain launches of this run so far
  bool chain_used = false;
  struct FStep {
    int step;
    float* dst;      // where the per-step path writes the state (a transient unit for intermediate steps)
    float* gates;
    bool wanted;     // a later launch reads this state; the others need not leave the chip
  };
  std::vector<FStep> fsteps;
  const std::vector<mebptt_op>& ops = plan->ops;

  // Before the first launch of this run that wants the whole chip: wait for the last run that had
  // such launches (on whatever stream), unless this stream is being captured.
  auto order_resident_launches = [&]() -> int {
    if (chain_used) return MEBPTT_OK;
    chain_used = true;
    int dev = 0;
    HIP_TRY(hipGetDevice(&dev));
    hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
    HIP_TRY(hipStreamIsCapturing(st, &cap));
    chain_order_dev = (cap == hipStreamCaptureStatusNone && dev >= 0 && dev < MAX_DEVICES) ? dev : -1;
    if (chain_order_dev >= 0 && g_chain_recorded[chain_order_dev])
      HIP_TRY(hipStreamWaitEvent(st, g_chain_done[chain_order_dev], 0));
    return MEBPTT_OK;
  };
  // "forward operation of step s keeping its internal state in the working core, then the backward
  // operation of step s" -- the pair every step of a sub-sequence that fits into memory ends in.
  const bool sweep_ok = resident_ok && can_run_sweep(d);
  auto pair_at = [&](size_t i) {
    if (i + 1 >= ops.size()) return false;
    const mebptt_op &f = ops[i], &b = ops[i + 1];
    return f.op == MEBPTT_OP_FWD_RUN && f.count == 1 && f.keep && f.dst == MEBPTT_LOC_CORE && b.op == MEBPTT_OP_BWD &&
           b.dst == MEBPTT_LOC_CORE && b.src == f.src && b.step == f.step;
  };

  // Where backward-only sweep launches exist but sweep launches with forward operations do not (the
  // weights of both directions do not fit on the chip together), runs of such pairs are recomputed
  // as a batch: see the main loop.  (The workspace has a stage exactly on those shapes.)
  const bool batch_ok = resident_ok && can_run_backward_sweep(d) && w.stage_steps >= 2;
  // Backward operations through internal states that earlier launches stored in slots (internal-state
  // pushes; store-everything BPTT): consecutive ones go out as backward-only sweep launches.
  const bool bsweep_ok = resident_ok && can_run_backward_sweep(d);
  auto stored_bwd_at = [&](size_t i) { return i < ops.size() && ops[i].op == MEBPTT_OP_BWD && ops[i].dst >= 0; };
  // One sweep launch for steps s_hi, s_hi - 1, ... (n of them, in one chunk or crossing from one into
  // the chunk below); states == nullptr: with forward operations.
  auto issue_sweep = [&](int s_hi, int n, const float* const* srcs, const float* const* states) -> int {
    const int chunk_hi = (s_hi - 1) / CH, chunk_lo = (s_hi - n) / CH;
    if (have_pending) {
      rc = flush_backward(nullptr, nullptr, nullptr, nullptr);
      if (rc) return rc;
    }
    for (int c = chunk_hi; c >= chunk_lo; --c) {   // the buffers of every chunk the launch writes into must be free
      rc = begin_chunk(c);
      if (rc) return rc;
    }
    rc = order_resident_launches();
    if (rc) return rc;
    SweepArgs a{};
    a.Wp = Wp;
    a.WTh = WTh;
    a.bp = bp;
    a.x = x;
    a.dy = desc->loss == 0 ? dy : nullptr;
    a.dy_first = desc->dy_first_step;
    a.dy_is_h = desc->loss == 1;
    a.dc = dc;
    a.y_out = y_out;
    a.dG_next = (s_hi == t) ? nullptr : ws + w.dG[(s_hi / CH) & 1] + (size_t)(s_hi % CH) * dG_step;
    for (int i = 0; i < 2; ++i) {
      a.dG_chunk[i] = ws + w.dG[i];
      a.dGT[i] = ws + w.dGT[i];
      a.aT[i] = ws + w.aT[i];
    }
    a.sync = reinterpret_cast<unsigned*>(ws + w.sync);
    a.base = chain_base;
    a.launch = chain_launches;
    a.s_hi = s_hi;
    a.count = n;
    a.src = srcs;
    a.state = states;
    rc = whole_launch(MEBPTT_K_SWEEP, n, st, [&] { return launch_sweep(d, a, st); });
    if (rc) return rc;
    if (use_profiler && g_prof.every_n > 0 && !states) g_prof.sweep_forward_steps += n;
    chain_base += forward_chain_arrivals(n);
    ++chain_launches;
    bwd += n;
    if (!states) fwd += n;
    for (int c = chunk_hi; c >= chunk_lo; --c)   // chunks whose first step the launch has back-propagated
      if (c * CH + 1 >= s_hi - n + 1) {
        rc = complete_chunk(c);
        if (rc) return rc;
      }
    return MEBPTT_OK;
  };

  const float* handed_src = nullptr;   // input state of a step a forward chain handed over to the next sweep launch
  int handed_step = 0;
  for (size_t oi = 0; oi < ops.size();) {
    const mebptt_op& op = ops[oi];
    if (bsweep_ok && stored_bwd_at(oi) && stored_bwd_at(oi + 1)) {
      const int s_hi = op.step, chunk = (s_hi - 1) / CH;
      int n = 0;
      const float *srcs[64], *states[64];
      const int reach = may_cross(chunk) ? 1 : 0;   // (store-everything BPTT: these launches follow each other directly)
      while (n < sweep_max_steps() && stored_bwd_at(oi + (size_t)n) && ops[oi + (size_t)n].step == s_hi - n &&
             chunk - (s_hi - n - 1) / CH <= reach) {
        srcs[n] = loc(ops[oi + (size_t)n].src);
        states[n] = loc(ops[oi + (size_t)n].dst);
        ++n;
      }
      if (n >= 2) {
        for (int j = 0; j < n; ++j) {
          touch(ops[oi + (size_t)j].dst, 3);
          touch(ops[oi + (size_t)j].src, 1);
        }
        rc = issue_sweep(s_hi, n, srcs, states);
        if (rc) return rc;
        oi += (size_t)n;
        continue;
      }
    }
    // A backward operation whose internal state a forward run has just left in the working core,
    // followed by such pairs for the steps below it, leads their launch: it is the first step of
    // the sweep launch, on the state in the core, the others on the states in the stage.
    const bool lead = batch_ok && op.op == MEBPTT_OP_BWD && op.dst == MEBPTT_LOC_CORE && pair_at(oi + 1) &&
                      ops[oi + 1].step == op.step - 1;
    if (batch_ok && (lead || pair_at(oi))) {
      // A run of such pairs for steps going down (in at most two chunks), every step's input state in a
      // slot: the forward operations do not depend on each other and go out as one launch that
      // leaves the internal states in the stage; one backward-only sweep launch then consumes them.
      const int s_hi = op.step, chunk = (s_hi - 1) / CH, nl = lead ? 1 : 0;
      const size_t first = oi + (size_t)nl;   // schedule entry of the first pair
      const int n_max = std::min(sweep_max_steps(), w.stage_steps) - nl;
      const int reach = may_cross(chunk) ? 1 : 0;   // chunks below the first the launch may run into
      int n = 0;   // pairs
      const float *srcs[64], *xs[64], *states[64];
      float* dsts[64];
      if (lead) {
        srcs[0] = loc(op.src);
        states[0] = loc(op.dst);
        xs[0] = nullptr;
        dsts[0] = nullptr;
      }
      while (n < n_max && pair_at(first + 2 * (size_t)n) && ops[first + 2 * (size_t)n].step == s_hi - nl - n &&
             ops[first + 2 * (size_t)n].src >= 0 && chunk - (s_hi - nl - n - 1) / CH <= reach) {
        srcs[nl + n] = loc(ops[first + 2 * (size_t)n].src);
        xs[nl + n] = x + (size_t)(s_hi - nl - n - 1) * d.B * d.I;
        dsts[nl + n] = reinterpret_cast<float*>(ws + w.stage) + (size_t)n * 3 * unit;
        states[nl + n] = dsts[nl + n];
        ++n;
      }
      if (n >= 1 && n + nl >= 2) {
        if (have_pending) {
          rc = flush_backward(nullptr, nullptr, nullptr, nullptr);
          if (rc) return rc;
        }
        if (lead) {
          touch(op.dst, 3);
          touch(op.src, 1);
        }
        for (int j = 0; j < n; ++j) touch(ops[first + 2 * (size_t)j].src, 1);
        rc = whole_launch(MEBPTT_K_FWD_BATCH, n, st,
                          [&] { return launch_forward_batch(d, Wp, bp, n, xs + nl, srcs + nl, dsts + nl, st); });
        if (rc) return rc;
        fwd += n;
        rc = issue_sweep(s_hi, n + nl, srcs, states);
        if (rc) return rc;
        oi = first + 2 * (size_t)n;
        continue;
      }
    }
    if (sweep_ok && (handed_src || pair_at(oi))) {
      // a run of such pairs for steps going down (in at most two chunks) goes out as one sweep launch,
      // starting with the step a forward chain handed over, if there is one (see below)
      const int nl = handed_src ? 1 : 0;
      const int s_hi = nl ? handed_step : op.step, chunk = (s_hi - 1) / CH;
      const int reach = may_cross(chunk) ? 1 : 0;
      int n = 0;   // pairs
      const float* srcs[64];
      srcs[0] = handed_src;
      while (n + nl < sweep_max_steps() && pair_at(oi + 2 * (size_t)n) && ops[oi + 2 * (size_t)n].step == s_hi - nl - n &&
             chunk - (s_hi - nl - n - 1) / CH <= reach) {
        srcs[nl + n] = loc(ops[oi + 2 * (size_t)n].src);
        ++n;
      }
      if (nl && n == 0) return set_error(MEBPTT_EINVAL, "internal: a handed-over step found no pair to join");
      if (n + nl >= 2) {
        for (int j = 0; j < n; ++j) touch(ops[oi + 2 * (size_t)j].src, 1);
        rc = issue_sweep(s_hi, n + nl, srcs, nullptr);
        if (rc) return rc;
        oi += 2 * (size_t)n;
        handed_src = nullptr;
        continue;
      }
    }
    if (op.op == MEBPTT_OP_FWD_RUN) {
      size_t oe = oi + 1;
      if (chain_ok)
        while (oe < ops.size() && ops[oe].op == MEBPTT_OP_FWD_RUN && ops[oe].src == ops[oe - 1].dst &&
               ops[oe - 1].dst != MEBPTT_LOC_CORE)
          ++oe;
      // Hand-over.  The last run of the chain would leave the internal state of its last step in the
      // core for the backward operation that follows, and pairs for the steps below follow that.  A
      // sweep launch recomputes internal states itself: the chain stops one step short (h of the step
      // before is where the run's `prev` puts it anyway) and the sweep launch starts one step
      // higher, at the handed-over step.  Every forward operation still runs exactly once.
      const mebptt_op& last = ops[oe - 1];
      const bool hand_over =
          sweep_ok && last.count >= 2 && last.keep && last.dst == MEBPTT_LOC_CORE && oe + 2 < ops.size() &&
          ops[oe].op == MEBPTT_OP_BWD && ops[oe].dst == MEBPTT_LOC_CORE && ops[oe].src == last.prev &&
          ops[oe].step == last.step + last.count - 1 && pair_at(oe + 1) && ops[oe + 1].step == ops[oe].step - 1;
      fsteps.clear();
      for (size_t k = oi; k < oe; ++k) {
        const mebptt_op& o = ops[k];
        const bool short_run = hand_over && k == oe - 1;   // its last step goes to the sweep launch
        if (o.dst == MEBPTT_LOC_CORE && !short_run) core_flip ^= 1;   // fresh core buffer: the held-back step may still read the other
        touch(o.src, 1);
        if (!short_run) touch(o.dst, o.keep ? 3 : 1);
        if (o.count > 1) touch(o.prev, 1);
        for (int j = 1; j <= o.count - (short_run ? 1 : 0); ++j) {
          float* dst = (j == o.count) ? loc(o.dst)
                                      : (j == o.count - 1 ? loc(o.prev) : loc((j & 1) ? MEBPTT_LOC_T1 : MEBPTT_LOC_T0));
          fsteps.push_back(FStep{o.step + j - 1, dst, (j == o.count && o.keep) ? dst + unit : nullptr, j >= o.count - 1});
        }
      }
      const float* cur = loc(op.src);
      size_t fi = 0;
      const size_t total = fsteps.size();
      auto x_of = [&](int step) { return x + (size_t)(step - 1) * d.B * d.I; };
      if (have_pending) {
        // units written by the first forward step vs units read by the held-back backward step
        const FStep& f = fsteps[0];
        const float* w_lo = f.dst;
        const float* w_hi = f.dst + (f.gates ? 3 : 1) * unit;
        const bool clash = (w_lo < pend.state + 3 * unit && pend.state < w_hi) ||
                           (w_lo < pend.prev + unit && pend.prev < w_hi);
        if (fuse && !clash) {
          rc = flush_backward(x_of(f.step), cur, f.dst, f.gates);
          if (rc) return rc;
          cur = f.dst;
          fi = 1;
        } else {
          rc = flush_backward(nullptr, nullptr, nullptr, nullptr);
          if (rc) return rc;
        }
      }
      if (chain_ok && total - fi >= (size_t)CHAIN_MIN_STEPS) {
        rc = order_resident_launches();
        if (rc) return rc;
        const int max_steps = forward_chain_max_steps();
        ChainStep cs[256];   // >= forward_chain_max_steps()
        while (fi < total) {
          const int n = (int)std::min<size_t>(total - fi, (size_t)max_steps);
          for (int j = 0; j < n; ++j) {
            const FStep& f = fsteps[fi + j];
            const bool keep_state = f.wanted || j == n - 1;   // the last state of a launch feeds the next launch
            cs[j] = ChainStep{keep_state ? f.dst : nullptr, f.gates};
          }
          const float* x_first = x_of(fsteps[fi].step);
          rc = whole_launch(MEBPTT_K_CHAIN, n, st, [&] {
            return launch_forward_chain(d, Wp, bp, x_first, cur, cs, n, ws + w.ring, reinterpret_cast<unsigned*>(ws + w.sync),
                                        chain_base, chain_launches, st);
          });
          if (rc) return rc;
          ++chain_launches;
          chain_base += forward_chain_arrivals(n);
          cur = fsteps[fi + n - 1].dst;
          fi += n;
          fwd += n;
        }
      } else {
        // Measurement hook: one event pair around the back-to-back launches of a long run.
        const bool bracket = use_profiler && g_prof.every_n > 0 && total - fi >= 8 && g_prof.runs.size() < 100000;
        Sample run_sample{MEBPTT_K_FORWARD, nullptr, nullptr, (int64_t)(total - fi)};
        if (bracket) {
          HIP_TRY(close_group());
          run_sample.start = g_prof.get();
          run_sample.stop = g_prof.get();
          if (!run_sample.start || !run_sample.stop) return set_error(MEBPTT_EHIP, "event creation failed");
          HIP_TRY(hipEventRecord(run_sample.start, st));
          g_prof.in_run = true;
        }
        for (; fi < total; ++fi) {
          const FStep& f = fsteps[fi];
          HIP_TRY(tm(MEBPTT_K_FORWARD, st, [&] { return launch_forward(d, Wp, bp, x_of(f.step), cur, f.dst, f.gates, st); }));
          cur = f.dst;
          ++fwd;
        }
        if (bracket) {
          g_prof.in_run = false;
          HIP_TRY(hipEventRecord(run_sample.stop, st));
          g_prof.runs.push_back(run_sample);
        }
      }
      if (hand_over) {
        handed_src = loc(last.prev);
        handed_step = ops[oe].step;
        oi = oe + 1;   // past the backward operation: the sweep launch carries it
      } else {
        oi = oe;
      }
      continue;
    } else if (op.op == MEBPTT_OP_BWD) {
      if (have_pending) {
        rc = flush_backward(nullptr, nullptr, nullptr, nullptr);
        if (rc) return rc;
      }
      const int s = op.step;
      const int chunk = (s - 1) / CH, slot = (s - 1) % CH, buf = chunk & 1;
      rc = begin_chunk(chunk);
      if (rc) return rc;
      touch(op.dst, 3);
      touch(op.src, 1);
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
    ++oi;
  }
  if (have_pending) {
    rc = flush_backward(nullptr, nullptr, nullptr, nullptr);
    if (rc) return rc;
  }
  // LSTM: dh_0 = dG_1 W_hh ; dc_0 is the running cell gradient after step 1.
  // GRU:  dh_0 = dG_1 W_hh + dh_1 * z_1 (the running plane) ; there is no cell state: dc_0 = 0.
  HIP_TRY(tm(MEBPTT_K_DGRAD, st, [&] { return launch_dgrad_gemm(d, WTh, d.H, ws + w.dG[0], 1, dh0, d.H, st); }));
  if (d.cell == MEBPTT_CELL_LSTM) {
    HIP_TRY(tm(MEBPTT_K_SETUP, st, [&] { return launch_copy_plane(d, dc, dc0, 0, st); }));
  } else {
    HIP_TRY(tm(MEBPTT_K_SETUP, st, [&] { return launch_copy_plane(d, dc, dh0, 1, st); }));
    HIP_TRY(launch_copy_plane(d, dc, dc0, 2, st));
  }
  for (int i = 0; i < 2; ++i)   // join: everything is ordered before whatever follows on `st`
    if (pending[i]) HIP_TRY(hipStreamWaitEvent(st, side->done[i], 0));
  HIP_TRY(tm(MEBPTT_K_WGRAD, st, [&] {
    return launch_wgrad_finish(d, reinterpret_cast<const float*>(ws + w.dWacc), dW_ih, dW_hh, db, st);
  }));

  if (use_profiler) HIP_TRY(close_group());
  if (chain_used && chain_order_dev >= 0) {
    if (!g_chain_done[chain_order_dev])
      HIP_TRY(hipEventCreateWithFlags(&g_chain_done[chain_order_dev], hipEventDisableTiming));
    HIP_TRY(hipEventRecord(g_chain_done[chain_order_dev], st));
    g_chain_recorded[chain_order_dev] = true;
  }

  if (stats) {
    stats->forward_ops = fwd;
    stats->backward_ops = bwd;
    stats->peak = (int32_t)((high_water + units_per_budget - 1) / units_per_budget);
    stats->reserved = 0;
    stats->peak_slot_bytes = (size_t)high_water * mebptt_unit_bytes(desc);
  }
  return MEBPTT_OK;
}

}  // namespace
