// Executor for a chain of non-homogeneous layers (appendix "Generalizing to deep feed-forward
// networks"): runs the schedule of a mebptt_chain_plan_t on a stack of dense tanh layers
//     y_i = tanh(y_{i-1} W_i^T + b_i),   W_i [d_i, d_{i-1}],   i = 1 .. n
// of differing widths, so that forward cost u_i = d_{i-1} d_i and state size s_i = B d_i differ from
// layer to layer.  Memorised outputs live in the caller's pool at the unit offsets the plan
// assigned; everything else (the two most recent activations of a forward run, the gradient being
// passed down, one layer's dz) is working memory in the caller's workspace, outside the budget.
//
// All three products of a layer are written as D[i][j] = sum_k A(i,k) B(k,j) with strided
// operands and executed by one kernel on fp32 MFMA tiles (v_mfma_f32_16x16x4_f32, fp32
// accumulate):
//   forward        y   [B, d_i]      = y_{i-1} [B, d_{i-1}] . W_i^T            then + b, tanh
//   backward data  g'  [B, d_{i-1}]  = dz [B, d_i] . W_i
//   backward weight dW [d_i, d_{i-1}] = dz^T . y_{i-1}                          (K = B)
// with dz = g * (1 - y_i^2) and db = column sums of dz.
#include <hip/hip_runtime.h>

#include <algorithm>
#include <vector>

#include "common.h"

using namespace mebptt;

namespace {

typedef __attribute__((ext_vector_type(4))) float f32x4;

enum { EPI_STORE = 0, EPI_BIAS_TANH = 1 };

// One wave per 16 x 16 output tile, four waves (2 x 2 tiles) per workgroup.
// A(i, k) = A[i * sai + k * sak], B(k, j) = Bm[k * sbk + j * sbj], C[i * ldc + j].
__global__ __launch_bounds__(256) void chain_gemm_kernel(const float* __restrict__ A, long sai, long sak,
                                                         const float* __restrict__ Bm, long sbk, long sbj,
                                                         float* __restrict__ C, long ldc, int M, int N, int K,
                                                         const float* __restrict__ bias, int epilogue) {
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), lane = threadIdx.x & 63;   // scalar: conditions on it are scalar branches (an MFMA under an empty lane mask would still execute)
  const int i0 = (blockIdx.y * 2 + (wave >> 1)) * 16, j0 = (blockIdx.x * 2 + (wave & 1)) * 16;
  if (i0 >= M || j0 >= N) return;   // whole wave
  const int li = lane & 15, lk = lane >> 4;
  const int ia = min(i0 + li, M - 1), jb = min(j0 + li, N - 1);   // clamped rows/columns are never stored
  const float* ap = A + (long)ia * sai;
  const float* bp = Bm + (long)jb * sbj;
  f32x4 acc = {0.f, 0.f, 0.f, 0.f};
  for (int k = 0; k < K; k += 4) {
    const int kk = k + lk;
    const float a = kk < K ? ap[(long)kk * sak] : 0.0f;
    const float b = kk < K ? bp[(long)kk * sbk] : 0.0f;
    acc = __builtin_amdgcn_mfma_f32_16x16x4f32(a, b, acc, 0, 0, 0);
  }
  // lane holds D[4 * (lane / 16) + r][lane % 16]
  const int j = j0 + li;
  if (j >= N) return;
  const float bj = (epilogue == EPI_BIAS_TANH && bias) ? bias[j] : 0.0f;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int i = i0 + 4 * lk + r;
    if (i >= M) continue;
    float v = acc[r];
    if (epilogue == EPI_BIAS_TANH) v = tanhf(v + bj);
    C[(long)i * ldc + j] = v;
  }
}

// dz = g * (1 - y^2), elementwise over B * d values.
__global__ void chain_dz_kernel(const float* __restrict__ g, const float* __restrict__ y, float* __restrict__ dz, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dz[i] = g[i] * (1.0f - y[i] * y[i]);
}

// db[j] = sum_b dz[b][j], rows added in order (one thread per column).
__global__ void chain_colsum_kernel(const float* __restrict__ dz, int B, int d, float* __restrict__ db) {
  const int j = blockIdx.x * blockDim.x + threadIdx.x;
  if (j >= d) return;
  float s = 0.0f;
  for (int b = 0; b < B; ++b) s += dz[(size_t)b * d + j];
  db[j] = s;
}

__global__ void chain_copy_kernel(const float* __restrict__ src, float* __restrict__ dst, size_t n) {
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

hipError_t gemm(const float* A, long sai, long sak, const float* Bm, long sbk, long sbj, float* C, long ldc, int M, int N,
                int K, const float* bias, int epilogue, hipStream_t st) {
  dim3 grid((N + 31) / 32, (M + 31) / 32), block(256);
  chain_gemm_kernel<<<grid, block, 0, st>>>(A, sai, sak, Bm, sbk, sbj, C, ldc, M, N, K, bias, epilogue);
  return hipGetLastError();
}

unsigned blocks_for(size_t n) { return (unsigned)std::min<size_t>((n + 255) / 256, 2048); }

constexpr size_t ALIGN = 256;
size_t align_up(size_t v) { return (v + ALIGN - 1) / ALIGN * ALIGN; }

int check_chain_desc(const mebptt_chain_desc* d) {
  if (!d) return set_error(MEBPTT_EINVAL, "desc is NULL");
  if (d->n < 1 || d->B < 1 || !d->widths) return set_error(MEBPTT_EINVAL, "a chain needs n >= 1 layers, B >= 1 and widths");
  for (int i = 0; i <= d->n; ++i)
    if (d->widths[i] < 1 || d->widths[i] > (1 << 20)) return set_error(MEBPTT_EINVAL, "width %d is out of range", i);
  if (d->unit_bytes < 4 || d->unit_bytes % 4) return set_error(MEBPTT_EINVAL, "unit_bytes must be a positive multiple of 4");
  return MEBPTT_OK;
}

size_t max_width(const mebptt_chain_desc* d) {
  int w = 0;
  for (int i = 0; i <= d->n; ++i) w = std::max(w, d->widths[i]);
  return (size_t)w;
}

#define HIP_TRY(expr)                                                                                 \
  do {                                                                                                \
    hipError_t e_ = (expr);                                                                           \
    if (e_ != hipSuccess) return set_error(MEBPTT_EHIP, "%s failed: %s", #expr, hipGetErrorString(e_)); \
  } while (0)

}  // namespace


extern "C" {

int mebptt_chain_layers(const mebptt_chain_desc* desc, mebptt_layer* out) {
  int rc = check_chain_desc(desc);
  if (rc) return rc;
  if (!out) return set_error(MEBPTT_EINVAL, "out is NULL");
  for (int i = 1; i <= desc->n; ++i) {
    out[i - 1].cost = (int64_t)desc->widths[i - 1] * desc->widths[i];
    const size_t bytes = (size_t)desc->B * desc->widths[i] * sizeof(float);
    out[i - 1].state_units = (int32_t)((bytes + desc->unit_bytes - 1) / desc->unit_bytes);
    out[i - 1].work_units = 0;   // working memory is the caller's workspace, outside the budget
  }
  return MEBPTT_OK;
}

size_t mebptt_chain_workspace_bytes(const mebptt_chain_desc* desc) {
  if (check_chain_desc(desc) != MEBPTT_OK) return 0;
  // two activations, two gradients, one dz, each of the widest layer
  return 5 * align_up((size_t)desc->B * max_width(desc) * sizeof(float));
}

int mebptt_chain_run(const mebptt_chain_desc* desc, const mebptt_chain_plan_t* plan, const float* const* W,
                     const float* const* b, const float* x0, const float* dy, void* pool, size_t pool_bytes,
                     void* workspace, size_t workspace_bytes, float* const* dW, float* const* db, float* dx0,
                     float* y_out, mebptt_chain_stats* stats, void* stream) {
  int rc = check_chain_desc(desc);
  if (rc) return rc;
  if (!plan) return set_error(MEBPTT_EINVAL, "plan is NULL");
  if (!W || !b || !x0 || !dy || !dW || !db) return set_error(MEBPTT_EINVAL, "a required pointer is NULL");
  const int n = desc->n, B = desc->B;
  for (int i = 0; i < n; ++i)
    if (!W[i] || !dW[i] || !db[i]) return set_error(MEBPTT_EINVAL, "layer %d: W, dW and db are required", i + 1);
  if (!workspace) return set_error(MEBPTT_EWORKSPACE, "workspace is NULL");
  if (workspace_bytes < mebptt_chain_workspace_bytes(desc))
    return set_error(MEBPTT_EWORKSPACE, "workspace has %zu bytes, %zu needed", workspace_bytes,
                     mebptt_chain_workspace_bytes(desc));
  if ((reinterpret_cast<uintptr_t>(workspace) | reinterpret_cast<uintptr_t>(pool)) & (ALIGN - 1))
    return set_error(MEBPTT_EWORKSPACE, "pool and workspace must be 256-byte aligned");
  size_t nops = 0;
  const mebptt_chain_op* ops = mebptt_chain_plan_schedule(plan, &nops);
  if (!ops || nops == 0) return set_error(MEBPTT_EINVAL, "the plan carries no schedule");

  // the plan must have been made for this chain: same layer count, state sizes that match the widths
  std::vector<mebptt_layer> layers(n);
  rc = mebptt_chain_layers(desc, layers.data());
  if (rc) return rc;
  {
    int32_t pn = 0;
    const mebptt_layer* pl = mebptt_chain_plan_layers(plan, &pn);
    if (pn != n) return set_error(MEBPTT_ESHAPE, "the plan is for %d layers, the descriptor has %d", pn, n);
    for (int i = 0; i < n; ++i)
      if (pl[i].cost != layers[i].cost || pl[i].state_units != layers[i].state_units || pl[i].work_units != layers[i].work_units)
        return set_error(MEBPTT_ESHAPE, "layer %d of the plan does not match the descriptor (see mebptt_chain_layers)", i + 1);
  }
  const size_t unit = desc->unit_bytes;
  // Host-side check of every location before anything is enqueued.
  int64_t high_water = 0;
  int backward_seen = 0;
  for (size_t k = 0; k < nops; ++k) {
    const mebptt_chain_op& o = ops[k];
    if (o.layer < 1 || o.count < 1 || o.layer + o.count - 1 > n) return set_error(MEBPTT_ESHAPE, "schedule names a layer outside the chain");
    if (o.op == MEBPTT_CHAIN_FORWARD) {
      if (o.src >= 0) {
        if (o.layer < 2) return set_error(MEBPTT_ESHAPE, "schedule reads a memorised state below the first layer");
        high_water = std::max<int64_t>(high_water, (int64_t)o.src + layers[o.layer - 2].state_units);
      } else if (o.src != MEBPTT_CHAIN_INPUT) {
        return set_error(MEBPTT_ESHAPE, "a forward run must start from the input or a memorised state");
      } else if (o.layer != 1) {
        return set_error(MEBPTT_ESHAPE, "only the first layer reads the network input");
      }
      if (o.dst >= 0)
        high_water = std::max<int64_t>(high_water, (int64_t)o.dst + layers[o.layer + o.count - 2].state_units);
      else if (o.dst != MEBPTT_CHAIN_WORKING)
        return set_error(MEBPTT_ESHAPE, "unknown destination %d", o.dst);
    } else if (o.op == MEBPTT_CHAIN_BACKWARD) {
      if (o.layer != n - backward_seen) return set_error(MEBPTT_ESHAPE, "backward operations out of order");
      ++backward_seen;
      if (o.src >= 0) {
        if (o.layer < 2) return set_error(MEBPTT_ESHAPE, "schedule reads a memorised state below the first layer");
        high_water = std::max<int64_t>(high_water, (int64_t)o.src + layers[o.layer - 2].state_units);
      } else if (o.src == MEBPTT_CHAIN_INPUT ? o.layer != 1 : o.src != MEBPTT_CHAIN_WORKING) {
        return set_error(MEBPTT_ESHAPE, "unknown source %d", o.src);
      }
    } else {
      return set_error(MEBPTT_EINVAL, "unknown schedule entry %d", o.op);
    }
  }
  if (backward_seen != n) return set_error(MEBPTT_ESHAPE, "the plan is for another number of layers");
  if (high_water > 0 && !pool) return set_error(MEBPTT_ENOMEM_SLOTS, "pool is NULL");
  if ((size_t)high_water * unit > pool_bytes)
    return set_error(MEBPTT_ENOMEM_SLOTS, "pool has %zu bytes, the schedule reaches %zu", pool_bytes, (size_t)high_water * unit);

  hipStream_t st = reinterpret_cast<hipStream_t>(stream);
  char* ws = reinterpret_cast<char*>(workspace);
  const size_t slab = align_up((size_t)B * max_width(desc) * sizeof(float));
  float* act[2] = {reinterpret_cast<float*>(ws), reinterpret_cast<float*>(ws + slab)};
  float* grad[2] = {reinterpret_cast<float*>(ws + 2 * slab), reinterpret_cast<float*>(ws + 3 * slab)};
  float* dz = reinterpret_cast<float*>(ws + 4 * slab);
  auto pool_at = [&](int32_t off) { return reinterpret_cast<float*>(reinterpret_cast<char*>(pool) + (size_t)off * unit); };

  // working memory after a forward run: `wk_out` = its last output, `wk_in` = the activation before it
  const float* wk_in = nullptr;
  const float* wk_out = nullptr;
  int flip = 0, gflip = 0;
  const float* g = dy;   // gradient with respect to the output of the layer about to be back-propagated
  int64_t forward_cost = 0, backward_ops = 0;

  for (size_t k = 0; k < nops; ++k) {
    const mebptt_chain_op& o = ops[k];
    if (o.op == MEBPTT_CHAIN_FORWARD) {
      const float* a = o.src == MEBPTT_CHAIN_INPUT ? x0 : pool_at(o.src);
      const float* before = nullptr;
      for (int i = 0; i < o.count; ++i) {
        const int L = o.layer + i;                         // 1-based layer
        const int din = desc->widths[L - 1], dout = desc->widths[L];
        const bool last = i == o.count - 1;
        float* out = (last && o.dst >= 0) ? pool_at(o.dst) : act[flip];
        if (!(last && o.dst >= 0)) flip ^= 1;
        // y [B, dout] = a [B, din] . W^T : A(i,k) = a[i*din + k], B(k,j) = W[j*din + k]
        HIP_TRY(gemm(a, din, 1, W[L - 1], 1, din, out, dout, B, dout, din, b[L - 1], EPI_BIAS_TANH, st));
        forward_cost += layers[L - 1].cost;
        before = a;
        a = out;
      }
      wk_in = before;
      wk_out = a;
      if (o.layer + o.count - 1 == n && y_out)
        chain_copy_kernel<<<blocks_for((size_t)B * desc->widths[n]), 256, 0, st>>>(a, y_out, (size_t)B * desc->widths[n]);
    } else {
      const int L = o.layer, din = desc->widths[L - 1], dout = desc->widths[L];
      const float* xin = o.src == MEBPTT_CHAIN_INPUT ? x0 : (o.src == MEBPTT_CHAIN_WORKING ? wk_in : pool_at(o.src));
      if (!wk_out || !xin) return set_error(MEBPTT_ESHAPE, "backward operation without a forward operation before it");
      const size_t ne = (size_t)B * dout;
      chain_dz_kernel<<<blocks_for(ne), 256, 0, st>>>(g, wk_out, dz, ne);
      HIP_TRY(hipGetLastError());
      chain_colsum_kernel<<<(dout + 255) / 256, 256, 0, st>>>(dz, B, dout, db[L - 1]);
      HIP_TRY(hipGetLastError());
      // dW [dout, din] = dz^T . x : A(i,k) = dz[k*dout + i], B(k,j) = x[k*din + j]
      HIP_TRY(gemm(dz, 1, dout, xin, din, 1, dW[L - 1], din, dout, din, B, nullptr, EPI_STORE, st));
      // g' [B, din] = dz . W : A(i,k) = dz[i*dout + k], B(k,j) = W[k*din + j]
      float* gout = (L == 1) ? dx0 : grad[gflip];
      if (gout) HIP_TRY(gemm(dz, dout, 1, W[L - 1], din, 1, gout, din, B, din, dout, nullptr, EPI_STORE, st));
      if (L > 1) {
        g = gout;
        gflip ^= 1;
      }
      ++backward_ops;
      wk_out = nullptr;   // consumed: the next backward operation needs its own forward operation
    }
  }
  if (stats) {
    stats->forward_cost = forward_cost;
    stats->backward_ops = backward_ops;
    stats->peak_units = (int32_t)high_water;
    stats->reserved = 0;
  }
  return MEBPTT_OK;
}

}  // extern "C"
