// HIP kernels for gfx950 (CDNA4, 64-wide wavefronts, MFMA matrix cores).
//
// Every contraction is written as D[i][j] = sum_k A[i][k] * B[j][k] with both operands
// k-contiguous in memory, and executed with 16x16 MFMA tiles:
//   bf16 operands: v_mfma_f32_16x16x32_bf16, each lane supplies 8 consecutive k of row lane%16
//   fp32 operands: v_mfma_f32_16x16x4_f32 issued 4 times over 4 consecutive k per lane
// so one "macro step" covers 4*VEC values of k (VEC = 8 or 4), lane group lane/16 owning the
// VEC-wide slice number lane/16.  (Which k a lane feeds is irrelevant as long as A and B agree.)
// The accumulator of lane l holds D[4*(l/16) + r][l%16], r = 0..3.
//
// The weights always play A (rows = gate rows or hidden units) and the batch plays B (columns),
// so a lane ends up with FOUR CONSECUTIVE ROWS of one batch column.  The forward operand is
// row-permuted so that those four rows are the gates i, f, g, o of one hidden unit: the LSTM
// pointwise step then runs entirely in registers (K1 + K2 of the hot path fused).  In the
// backward step the four rows are four consecutive hidden units of dh, and the pointwise
// backward (K3 + K4) again runs in registers on the GEMM result (K5's dh half fused with K4 of
// the next step down).
#include "kernels.h"

namespace mebptt {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

Dims make_dims(int B, int I, int H, int dtype) {
  Dims d{};
  d.B = B;
  d.I = I;
  d.H = H;
  d.dtype = dtype;
  d.HP = round_up(H, 16);
  d.KX = round_up(I, 32);
  d.KH = round_up(H, 32);
  d.KP = d.KX + d.KH;
  d.NX = round_up(I, 16);
  d.BP = round_up(B, 16);
  d.G4 = 4 * d.HP;
  int ch = 512 / B;   // aim at K ~ 512 for the weight-gradient GEMM
  d.CH = ch < 1 ? 1 : (ch > 32 ? 32 : ch);
  d.KC = round_up(d.CH * B, 32);
  return d;
}

// ---- operand traits ------------------------------------------------------------------------

template <class T>
struct Mma;

template <>
struct Mma<__bf16> {
  static constexpr int VEC = 8;
  using Frag = bf16x8;
  __device__ static Frag load(const __bf16* p) { return *reinterpret_cast<const Frag*>(p); }
  __device__ static Frag from_f32(const float (&v)[8]) {
    Frag f;
#pragma unroll
    for (int e = 0; e < 8; ++e) f[e] = (__bf16)v[e];
    return f;
  }
  __device__ static f32x4 mma(Frag a, Frag b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
};

template <>
struct Mma<float> {
  static constexpr int VEC = 4;
  using Frag = f32x4;
  __device__ static Frag load(const float* p) { return *reinterpret_cast<const Frag*>(p); }
  __device__ static Frag from_f32(const float (&v)[4]) { return Frag{v[0], v[1], v[2], v[3]}; }
  __device__ static f32x4 mma(Frag a, Frag b, f32x4 c) {
#pragma unroll
    for (int e = 0; e < 4; ++e) c = __builtin_amdgcn_mfma_f32_16x16x4f32(a[e], b[e], c, 0, 0, 0);
    return c;
  }
};

// VEC consecutive fp32 values row[k .. k+VEC), zero beyond `limit`, converted to the operand type.
template <class T>
__device__ inline typename Mma<T>::Frag load_act(const float* __restrict__ row, int k, int limit, bool vec_ok) {
  constexpr int VEC = Mma<T>::VEC;
  float v[VEC];
  if (vec_ok && k + VEC <= limit) {
#pragma unroll
    for (int e = 0; e < VEC; e += 4) {
      float4 q = *reinterpret_cast<const float4*>(row + k + e);
      v[e] = q.x;
      v[e + 1] = q.y;
      v[e + 2] = q.z;
      v[e + 3] = q.w;
    }
  } else {
#pragma unroll
    for (int e = 0; e < VEC; ++e) v[e] = (k + e < limit) ? row[k + e] : 0.0f;
  }
  return Mma<T>::from_f32(v);
}

__device__ inline float sigmoidf_(float z) { return 1.0f / (1.0f + expf(-z)); }

// ---- small utility kernels -------------------------------------------------------------------

__global__ void fill_zero_kernel(uint4* p, size_t n16) {
  size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (; i < n16; i += stride) p[i] = uint4{0, 0, 0, 0};
}

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st) {
  if (bytes == 0) return hipSuccess;
  size_t n16 = bytes / 16;   // callers keep every buffer a multiple of 16 bytes
  size_t blocks = (n16 + 255) / 256;
  if (blocks > 4096) blocks = 4096;
  fill_zero_kernel<<<dim3((unsigned)blocks), dim3(256), 0, st>>>(reinterpret_cast<uint4*>(p), n16);
  return hipGetLastError();
}

template <class T>
__global__ void prep_weights_kernel(Dims d, const float* __restrict__ W_ih, const float* __restrict__ W_hh,
                                    const float* __restrict__ b, T* __restrict__ Wp, float* __restrict__ bp,
                                    T* __restrict__ WTh, T* __restrict__ WTx) {
  const size_t nWp = (size_t)d.G4 * d.KP, nWTh = (size_t)d.HP * d.G4, nWTx = (size_t)d.NX * d.G4;
  const size_t total = nWp + nWTh + nWTx + (size_t)d.G4;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
    if (idx < nWp) {   // Wp[row'][k], row' = 4u + gate
      int rowp = (int)(idx / d.KP), k = (int)(idx % d.KP);
      int u = rowp >> 2, gate = rowp & 3;
      float v = 0.0f;
      if (u < d.H) {
        size_t row = (size_t)gate * d.H + u;
        if (k < d.KX) {
          if (k < d.I) v = W_ih[row * d.I + k];
        } else if (k - d.KX < d.H) {
          v = W_hh[row * d.H + (k - d.KX)];
        }
      }
      Wp[idx] = (T)v;
    } else if (idx < nWp + nWTh + nWTx) {   // WTh[n][4u+gate] / WTx[n][4u+gate]
      size_t j = idx - nWp;
      bool is_h = j < nWTh;
      if (!is_h) j -= nWTh;
      int n = (int)(j / d.G4), kp = (int)(j % d.G4);
      int u = kp >> 2, gate = kp & 3;
      float v = 0.0f;
      if (u < d.H) {
        size_t row = (size_t)gate * d.H + u;
        if (is_h) {
          if (n < d.H) v = W_hh[row * d.H + n];
        } else {
          if (n < d.I) v = W_ih[row * d.I + n];
        }
      }
      (is_h ? WTh : WTx)[j] = (T)v;
    } else {
      int kp = (int)(idx - nWp - nWTh - nWTx);
      int u = kp >> 2, gate = kp & 3;
      bp[kp] = (b != nullptr && u < d.H) ? b[(size_t)gate * d.H + u] : 0.0f;
    }
  }
}

hipError_t launch_prep_weights(const Dims& d, const float* W_ih, const float* W_hh, const float* b, void* Wp,
                               float* bp, void* WTh, void* WTx, hipStream_t st) {
  dim3 grid(2048), block(256);
  if (d.dtype)
    prep_weights_kernel<__bf16><<<grid, block, 0, st>>>(d, W_ih, W_hh, b, (__bf16*)Wp, bp, (__bf16*)WTh, (__bf16*)WTx);
  else
    prep_weights_kernel<float><<<grid, block, 0, st>>>(d, W_ih, W_hh, b, (float*)Wp, bp, (float*)WTh, (float*)WTx);
  return hipGetLastError();
}

__global__ void init_state_kernel(size_t n, const float* __restrict__ h0, const float* __restrict__ c0,
                                  float* __restrict__ dst) {
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    dst[i] = h0 ? h0[i] : 0.0f;
    dst[n + i] = c0 ? c0[i] : 0.0f;
  }
}

hipError_t launch_init_state(const Dims& d, const float* h0, const float* c0, float* dst_unit, hipStream_t st) {
  size_t n = (size_t)d.B * d.H;
  size_t blocks = (n + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  init_state_kernel<<<dim3((unsigned)blocks), dim3(256), 0, st>>>(n, h0, c0, dst_unit);
  return hipGetLastError();
}

__global__ void copy_plane_kernel(size_t n, const float* __restrict__ src, float* __restrict__ dst) {
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) dst[i] = src[i];
}

hipError_t launch_copy_plane(const Dims& d, const float* src, float* dst, hipStream_t st) {
  size_t n = (size_t)d.B * d.H;
  size_t blocks = (n + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  copy_plane_kernel<<<dim3((unsigned)blocks), dim3(256), 0, st>>>(n, src, dst);
  return hipGetLastError();
}

// ---- forward step: gate GEMM + LSTM pointwise -------------------------------------------------

struct FwdParams {
  const void* Wp;
  const float* bp;
  const float* x_s;
  const float* src_h;
  const float* src_c;
  float* dst_h;
  float* dst_c;
  float* g_i;   // NULL: do not keep the gates
  float* g_f;
  float* g_g;
  float* g_o;
  int B, I, H, HP, KX, KP;
};

// Workgroup = BT batch tiles x KS k-slices (one wave each); every wave covers NG unit groups
// (16 gate rows = 4 hidden units each) and reuses its activation fragment across them.
template <class T, int NG, int BT, int KS>
__global__ __launch_bounds__(64 * BT * KS) void forward_kernel(FwdParams p) {
  using M = Mma<T>;
  constexpr int VEC = M::VEC, KSTEP = 4 * VEC;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int bt = wave % BT, ks = wave / BT;
  const int lrow = lane & 15, lq = lane >> 4;
  const int group0 = blockIdx.x * NG;
  const int ngroups = p.HP >> 2;
  const int b0 = (blockIdx.y * BT + bt) * 16;
  const int b_ld = min(b0 + lrow, p.B - 1);
  const float* xrow = p.x_s + (size_t)b_ld * p.I;
  const float* hrow = p.src_h + (size_t)b_ld * p.H;
  const bool x_vec = (p.I & 3) == 0, h_vec = (p.H & 3) == 0;
  const T* wrow[NG];
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    int grp = min(group0 + g, ngroups - 1);
    wrow[g] = reinterpret_cast<const T*>(p.Wp) + ((size_t)grp * 16 + lrow) * p.KP + VEC * lq;
  }
  f32x4 acc[NG];
#pragma unroll
  for (int g = 0; g < NG; ++g) acc[g] = f32x4{0.f, 0.f, 0.f, 0.f};

  const int nsteps = p.KP / KSTEP;
  for (int s = ks; s < nsteps; s += KS) {
    const int k = s * KSTEP + VEC * lq;
    typename M::Frag bf = (k < p.KX) ? load_act<T>(xrow, k, p.I, x_vec) : load_act<T>(hrow, k - p.KX, p.H, h_vec);
#pragma unroll
    for (int g = 0; g < NG; ++g) {
      typename M::Frag af = M::load(wrow[g] + (size_t)s * KSTEP);
      acc[g] = M::mma(af, bf, acc[g]);
    }
  }

  if (KS > 1) {
    __shared__ float red[(KS > 1 ? KS - 1 : 1) * BT * NG * 4 * 64];
    if (ks > 0) {
#pragma unroll
      for (int g = 0; g < NG; ++g)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[((((ks - 1) * BT + bt) * NG + g) * 4 + r) * 64 + lane] = acc[g][r];
    }
    __syncthreads();
    if (ks == 0) {
      for (int q = 1; q < KS; ++q)   // fixed order: results do not depend on scheduling
#pragma unroll
        for (int g = 0; g < NG; ++g)
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[g][r] += red[((((q - 1) * BT + bt) * NG + g) * 4 + r) * 64 + lane];
    }
  }
  if (ks != 0) return;

  const int b = b0 + lrow;
  if (b >= p.B) return;
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    const int u = (group0 + g) * 4 + lq;
    if (u >= p.H) continue;
    const float4 bias = *reinterpret_cast<const float4*>(p.bp + 4 * u);
    const size_t e = (size_t)b * p.H + u;
    const float gi = sigmoidf_(acc[g][0] + bias.x);
    const float gf = sigmoidf_(acc[g][1] + bias.y);
    const float gg = tanhf(acc[g][2] + bias.z);
    const float go = sigmoidf_(acc[g][3] + bias.w);
    const float c = gf * p.src_c[e] + gi * gg;
    const float h = go * tanhf(c);
    p.dst_h[e] = h;
    p.dst_c[e] = c;
    if (p.g_i) {
      p.g_i[e] = gi;
      p.g_f[e] = gf;
      p.g_g[e] = gg;
      p.g_o[e] = go;
    }
  }
}

template <class T, int NG, int BT, int KS>
static hipError_t launch_forward_cfg(const Dims& d, const FwdParams& p, hipStream_t st) {
  dim3 grid((d.HP / 4 + NG - 1) / NG, (d.BP / 16 + BT - 1) / BT), block(64 * BT * KS);
  forward_kernel<T, NG, BT, KS><<<grid, block, 0, st>>>(p);
  return hipGetLastError();
}

template <class T>
static hipError_t launch_forward_t(const Dims& d, const FwdParams& p, hipStream_t st) {
  const int btiles = d.BP / 16;
  if (btiles >= 4) {
    // Large hidden sizes: two unit groups per wave halve the activation traffic per gate row.
    if ((size_t)d.HP / 4 * ((btiles + 3) / 4) >= 2048) return launch_forward_cfg<T, 2, 4, 4>(d, p, st);
    return launch_forward_cfg<T, 1, 4, 4>(d, p, st);
  }
  if (btiles >= 2) return launch_forward_cfg<T, 1, 2, 8>(d, p, st);
  return launch_forward_cfg<T, 1, 1, 8>(d, p, st);
}

hipError_t launch_forward(const Dims& d, const void* Wp, const float* bp, const float* x_s, const float* src_unit,
                          float* dst_unit, float* gates_units, hipStream_t st) {
  const size_t plane = (size_t)d.B * d.H;
  FwdParams p{};
  p.Wp = Wp;
  p.bp = bp;
  p.x_s = x_s;
  p.src_h = src_unit;
  p.src_c = src_unit + plane;
  p.dst_h = dst_unit;
  p.dst_c = dst_unit + plane;
  if (gates_units) {
    p.g_i = gates_units;
    p.g_f = gates_units + plane;
    p.g_g = gates_units + 2 * plane;
    p.g_o = gates_units + 3 * plane;
  }
  p.B = d.B;
  p.I = d.I;
  p.H = d.H;
  p.HP = d.HP;
  p.KX = d.KX;
  p.KP = d.KP;
  return d.dtype ? launch_forward_t<__bf16>(d, p, st) : launch_forward_t<float>(d, p, st);
}

// ---- backward step: dh GEMM + loss-gradient injection + LSTM pointwise backward --------------

struct BwdParams {
  const void* WTh;
  const void* dG_next;
  const float *h, *c, *g_i, *g_f, *g_g, *g_o, *h_prev, *c_prev, *dy_s;
  int dy_is_h;
  float* dc;
  void* dG_cur;
  void* dGT;
  void* aT;
  int col0;
  float* y_out_s;
  int B, H, HP, G4, NX, KC, BP;
};

// Workgroup = one tile of 16 hidden units x BT batch tiles x KS k-slices.
template <class T, int BT, int KS>
__global__ __launch_bounds__(64 * BT * KS) void backward_kernel(BwdParams p) {
  using M = Mma<T>;
  constexpr int VEC = M::VEC, KSTEP = 4 * VEC;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int bt = wave % BT, ks = wave / BT;
  const int lrow = lane & 15, lq = lane >> 4;
  const int n0 = blockIdx.x * 16;
  const int b0 = (blockIdx.y * BT + bt) * 16;
  f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
  if (p.dG_next) {
    const int brow = min(b0 + lrow, p.BP - 1);
    const T* arow = reinterpret_cast<const T*>(p.WTh) + (size_t)(n0 + lrow) * p.G4 + VEC * lq;
    const T* brow_p = reinterpret_cast<const T*>(p.dG_next) + (size_t)brow * p.G4 + VEC * lq;
    const int nsteps = p.G4 / KSTEP;
    for (int s = ks; s < nsteps; s += KS) {
      typename M::Frag af = M::load(arow + (size_t)s * KSTEP);
      typename M::Frag bf = M::load(brow_p + (size_t)s * KSTEP);
      acc = M::mma(af, bf, acc);
    }
    if (KS > 1) {
      __shared__ float red[(KS > 1 ? KS - 1 : 1) * BT * 4 * 64];
      if (ks > 0) {
#pragma unroll
        for (int r = 0; r < 4; ++r) red[(((ks - 1) * BT + bt) * 4 + r) * 64 + lane] = acc[r];
      }
      __syncthreads();
      if (ks == 0) {
        for (int q = 1; q < KS; ++q)
#pragma unroll
          for (int r = 0; r < 4; ++r) acc[r] += red[(((q - 1) * BT + bt) * 4 + r) * 64 + lane];
      }
    }
  }
  if (ks != 0) return;
  const int b = b0 + lrow;
  if (b >= p.B) return;
  T* dG_row = reinterpret_cast<T*>(p.dG_cur) + (size_t)b * p.G4;
  T* dGT = reinterpret_cast<T*>(p.dGT);
  T* aT = reinterpret_cast<T*>(p.aT);
  const int col = p.col0 + b;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int n = n0 + 4 * lq + r;
    if (n >= p.H) continue;
    const size_t e = (size_t)b * p.H + n;
    const float h = (p.dy_is_h || p.y_out_s) ? p.h[e] : 0.0f;
    float dh = acc[r];
    if (p.dy_is_h)
      dh += h;
    else if (p.dy_s)
      dh += p.dy_s[e];
    if (p.y_out_s) p.y_out_s[e] = h;
    const float gi = p.g_i[e], gf = p.g_f[e], gg = p.g_g[e], go = p.g_o[e];
    const float tc = tanhf(p.c[e]);
    const float c_prev = p.c_prev[e];
    const float d_o = dh * tc;
    const float dct = p.dc[e] + dh * go * (1.0f - tc * tc);
    const float dGi = dct * gg * gi * (1.0f - gi);
    const float dGf = dct * c_prev * gf * (1.0f - gf);
    const float dGg = dct * gi * (1.0f - gg * gg);
    const float dGo = d_o * go * (1.0f - go);
    p.dc[e] = dct * gf;
    const T q0 = (T)dGi, q1 = (T)dGf, q2 = (T)dGg, q3 = (T)dGo;
    dG_row[4 * n + 0] = q0;
    dG_row[4 * n + 1] = q1;
    dG_row[4 * n + 2] = q2;
    dG_row[4 * n + 3] = q3;
    dGT[(size_t)(4 * n + 0) * p.KC + col] = q0;
    dGT[(size_t)(4 * n + 1) * p.KC + col] = q1;
    dGT[(size_t)(4 * n + 2) * p.KC + col] = q2;
    dGT[(size_t)(4 * n + 3) * p.KC + col] = q3;
    aT[(size_t)(p.NX + n) * p.KC + col] = (T)p.h_prev[e];
  }
}

template <class T>
static hipError_t launch_backward_t(const Dims& d, const BwdParams& p, hipStream_t st) {
  const int btiles = d.BP / 16;
  if (btiles >= 4) {
    dim3 grid(d.HP / 16, (btiles + 3) / 4);
    backward_kernel<T, 4, 4><<<grid, dim3(1024), 0, st>>>(p);
  } else if (btiles >= 2) {
    dim3 grid(d.HP / 16, (btiles + 1) / 2);
    backward_kernel<T, 2, 8><<<grid, dim3(1024), 0, st>>>(p);
  } else {
    dim3 grid(d.HP / 16, btiles);
    backward_kernel<T, 1, 8><<<grid, dim3(512), 0, st>>>(p);
  }
  return hipGetLastError();
}

hipError_t launch_backward(const Dims& d, const BackwardArgs& a, hipStream_t st) {
  const size_t plane = (size_t)d.B * d.H;
  BwdParams p{};
  p.WTh = a.WTh;
  p.dG_next = a.dG_next;
  p.h = a.state;
  p.c = a.state + plane;
  p.g_i = a.state + 2 * plane;
  p.g_f = a.state + 3 * plane;
  p.g_g = a.state + 4 * plane;
  p.g_o = a.state + 5 * plane;
  p.h_prev = a.prev;
  p.c_prev = a.prev + plane;
  p.dy_s = a.dy_s;
  p.dy_is_h = a.dy_is_h;
  p.dc = a.dc;
  p.dG_cur = a.dG_cur;
  p.dGT = a.dGT;
  p.aT = a.aT;
  p.col0 = a.col0;
  p.y_out_s = a.y_out_s;
  p.B = d.B;
  p.H = d.H;
  p.HP = d.HP;
  p.G4 = d.G4;
  p.NX = d.NX;
  p.KC = d.KC;
  p.BP = d.BP;
  return d.dtype ? launch_backward_t<__bf16>(d, p, st) : launch_backward_t<float>(d, p, st);
}

// ---- data-gradient GEMM: out[row][n] = sum_k dG[row][k] * WT[n][k] ---------------------------

template <class T, int BT, int KS>
__global__ __launch_bounds__(64 * BT * KS) void dgrad_kernel(const T* __restrict__ WT, int N, const T* __restrict__ dG,
                                                             int nrows_padded, int B, int BP, int G4,
                                                             float* __restrict__ out, int ld_out) {
  using M = Mma<T>;
  constexpr int VEC = M::VEC, KSTEP = 4 * VEC;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int bt = wave % BT, ks = wave / BT;
  const int lrow = lane & 15, lq = lane >> 4;
  const int n0 = blockIdx.x * 16;
  const int r0 = (blockIdx.y * BT + bt) * 16;
  const int row_ld = min(r0 + lrow, nrows_padded - 1);
  const T* arow = WT + (size_t)(n0 + lrow) * G4 + VEC * lq;
  const T* brow = dG + (size_t)row_ld * G4 + VEC * lq;
  f32x4 acc = f32x4{0.f, 0.f, 0.f, 0.f};
  const int nsteps = G4 / KSTEP;
  for (int s = ks; s < nsteps; s += KS) {
    typename M::Frag af = M::load(arow + (size_t)s * KSTEP);
    typename M::Frag bf = M::load(brow + (size_t)s * KSTEP);
    acc = M::mma(af, bf, acc);
  }
  if (KS > 1) {
    __shared__ float red[(KS > 1 ? KS - 1 : 1) * BT * 4 * 64];
    if (ks > 0) {
#pragma unroll
      for (int r = 0; r < 4; ++r) red[(((ks - 1) * BT + bt) * 4 + r) * 64 + lane] = acc[r];
    }
    __syncthreads();
    if (ks == 0) {
      for (int q = 1; q < KS; ++q)
#pragma unroll
        for (int r = 0; r < 4; ++r) acc[r] += red[(((q - 1) * BT + bt) * 4 + r) * 64 + lane];
    }
  }
  if (ks != 0) return;
  const int row = r0 + lrow;
  if (row >= nrows_padded) return;
  const int slot = row / BP, b = row % BP;
  if (b >= B) return;
  float* orow = out + ((size_t)slot * B + b) * ld_out;
#pragma unroll
  for (int r = 0; r < 4; ++r) {
    const int n = n0 + 4 * lq + r;
    if (n < N) orow[n] = acc[r];
  }
}

hipError_t launch_dgrad_gemm(const Dims& d, const void* WT, int N, const void* dG, int nslots, float* out, int ld_out,
                             hipStream_t st) {
  const int nrows = nslots * d.BP;
  const int ntiles = round_up(N, 16) / 16, rtiles = nrows / 16;
  dim3 grid(ntiles, (rtiles + 3) / 4);
  if (d.dtype)
    dgrad_kernel<__bf16, 4, 4><<<grid, dim3(1024), 0, st>>>((const __bf16*)WT, N, (const __bf16*)dG, nrows, d.B, d.BP,
                                                            d.G4, out, ld_out);
  else
    dgrad_kernel<float, 4, 4><<<grid, dim3(1024), 0, st>>>((const float*)WT, N, (const float*)dG, nrows, d.B, d.BP, d.G4,
                                                           out, ld_out);
  return hipGetLastError();
}

// ---- x transposed into the weight-gradient operand ----------------------------------------------

template <class T>
__global__ void transpose_x_kernel(const float* __restrict__ x, int rows, int I, int KC, T* __restrict__ aT) {
  // x: [rows][I] (rows = nslots*B consecutive (step, b) pairs) -> aT[i][row]
  __shared__ float tile[32][33];
  const int r0 = blockIdx.x * 32, i0 = blockIdx.y * 32;
  const int tx = threadIdx.x & 31, ty = threadIdx.x >> 5;   // 32 x 8
  for (int rr = ty; rr < 32; rr += 8) {
    int r = r0 + rr, i = i0 + tx;
    tile[rr][tx] = (r < rows && i < I) ? x[(size_t)r * I + i] : 0.0f;
  }
  __syncthreads();
  for (int ii = ty; ii < 32; ii += 8) {
    int i = i0 + ii, r = r0 + tx;
    if (i < I && r < rows) aT[(size_t)i * KC + r] = (T)tile[tx][ii];
  }
}

hipError_t launch_transpose_x(const Dims& d, const float* x_first, int nslots, void* aT, hipStream_t st) {
  const int rows = nslots * d.B;
  dim3 grid((rows + 31) / 32, (d.I + 31) / 32), block(256);
  if (d.dtype)
    transpose_x_kernel<__bf16><<<grid, block, 0, st>>>(x_first, rows, d.I, d.KC, (__bf16*)aT);
  else
    transpose_x_kernel<float><<<grid, block, 0, st>>>(x_first, rows, d.I, d.KC, (float*)aT);
  return hipGetLastError();
}

// ---- weight-gradient GEMM: dW[row(m)][n] (+)= sum_k dGT[m][k] * aT[n][k] ------------------------

// Each wave owns a 64 x 64 block (4 x 4 MFMA tiles); a workgroup is 2 x 2 waves.
template <class T>
__global__ __launch_bounds__(256) void wgrad_kernel(const T* __restrict__ dGT, const T* __restrict__ aT, int K, int KC,
                                                    int G4, int NTOT, int NX, int I, int H, int accumulate,
                                                    float* __restrict__ dW_ih, float* __restrict__ dW_hh) {
  using M = Mma<T>;
  constexpr int VEC = M::VEC, KSTEP = 4 * VEC;
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int lrow = lane & 15, lq = lane >> 4;
  const int mt0 = (blockIdx.x * 2 + (wave & 1)) * 4;    // first 16-row tile of this wave
  const int nt0 = (blockIdx.y * 2 + (wave >> 1)) * 4;
  const int MT = G4 / 16, NT = NTOT / 16;
  if (mt0 >= MT || nt0 >= NT) return;
  const T* ap[4];
  const T* bp[4];
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    int mt = min(mt0 + i, MT - 1), nt = min(nt0 + i, NT - 1);
    ap[i] = dGT + (size_t)(mt * 16 + lrow) * KC + VEC * lq;
    bp[i] = aT + (size_t)(nt * 16 + lrow) * KC + VEC * lq;
  }
  f32x4 acc[4][4];
#pragma unroll
  for (int i = 0; i < 4; ++i)
#pragma unroll
    for (int j = 0; j < 4; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int k = 0; k < K; k += KSTEP) {
    typename M::Frag af[4], bf[4];
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      af[i] = M::load(ap[i] + k);
      bf[i] = M::load(bp[i] + k);
    }
#pragma unroll
    for (int i = 0; i < 4; ++i)
#pragma unroll
      for (int j = 0; j < 4; ++j) acc[i][j] = M::mma(af[i], bf[j], acc[i][j]);
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    if (mt0 + i >= MT) continue;
    const int u = (mt0 + i) * 4 + lq;   // permuted row 4u + gate, gate = r
    if (u >= H) continue;
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      if (nt0 + j >= NT) continue;
      const int n = (nt0 + j) * 16 + lrow;
#pragma unroll
      for (int r = 0; r < 4; ++r) {
        const size_t row = (size_t)r * H + u;
        float* dst;
        if (n < NX) {
          if (n >= I) continue;
          dst = dW_ih + row * I + n;
        } else {
          if (n - NX >= H) continue;
          dst = dW_hh + row * H + (n - NX);
        }
        *dst = accumulate ? (*dst + acc[i][j][r]) : acc[i][j][r];
      }
    }
  }
}

template <class T>
__global__ __launch_bounds__(256) void bias_grad_kernel(const T* __restrict__ dGT, int K, int KC, int G4, int H,
                                                        int accumulate, float* __restrict__ db) {
  const int wave = threadIdx.x >> 6, lane = threadIdx.x & 63;
  const int m = blockIdx.x * 4 + wave;
  if (m >= G4) return;
  const int u = m >> 2, gate = m & 3;
  if (u >= H) return;
  float s = 0.0f;
  for (int k = lane; k < K; k += 64) s += (float)dGT[(size_t)m * KC + k];
#pragma unroll
  for (int off = 32; off > 0; off >>= 1) s += __shfl_down(s, off, 64);
  if (lane == 0) {
    float* dst = db + (size_t)gate * H + u;
    *dst = accumulate ? (*dst + s) : s;
  }
}

hipError_t launch_wgrad(const Dims& d, const void* dGT, const void* aT, int nslots, int accumulate, float* dW_ih,
                        float* dW_hh, float* db, hipStream_t st) {
  const int kstep = d.dtype ? 32 : 16;
  const int K = round_up(nslots * d.B, kstep);   // columns past nslots*B are zero
  const int NTOT = d.NX + d.HP;
  dim3 grid((d.G4 / 16 + 7) / 8, (NTOT / 16 + 7) / 8), block(256);
  dim3 bgrid((d.G4 + 3) / 4);
  if (d.dtype) {
    wgrad_kernel<__bf16><<<grid, block, 0, st>>>((const __bf16*)dGT, (const __bf16*)aT, K, d.KC, d.G4, NTOT, d.NX, d.I,
                                                 d.H, accumulate, dW_ih, dW_hh);
    bias_grad_kernel<__bf16><<<bgrid, block, 0, st>>>((const __bf16*)dGT, nslots * d.B, d.KC, d.G4, d.H, accumulate, db);
  } else {
    wgrad_kernel<float><<<grid, block, 0, st>>>((const float*)dGT, (const float*)aT, K, d.KC, d.G4, NTOT, d.NX, d.I, d.H,
                                                accumulate, dW_ih, dW_hh);
    bias_grad_kernel<float><<<bgrid, block, 0, st>>>((const float*)dGT, nslots * d.B, d.KC, d.G4, d.H, accumulate, db);
  }
  return hipGetLastError();
}

}  // namespace mebptt
