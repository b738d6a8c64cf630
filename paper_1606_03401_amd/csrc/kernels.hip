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
// pointwise step then runs on the GEMM result without leaving the workgroup (gate GEMM and
// pointwise forward fused).  In the backward step the four rows are four consecutive hidden
// units of dh, and loss-gradient injection and the pointwise backward again run on the GEMM
// result (the dh = dG W_hh product of step s+1 fused with the pointwise backward of step s).
#include <type_traits>

#include "kernels.h"

namespace mebptt {

typedef __attribute__((ext_vector_type(8))) __bf16 bf16x8;
typedef __attribute__((ext_vector_type(4))) float f32x4;

Dims make_dims(int B, int I, int H, int dtype, int cell) {
  Dims d{};
  d.cell = cell;
  d.B = B;
  d.I = I;
  d.H = H;
  d.dtype = dtype;
  d.HP = round_up(H, dtype ? 32 : 16);   // bf16: HP == KH, so every column of a split h plane belongs to a tile
  d.KX = round_up(I, 32);
  d.KH = round_up(H, 32);
  d.KP = d.KX + d.KH;
  d.NX = round_up(I, 16);
  d.BP = round_up(B, 16);
  d.G4 = 4 * d.HP;
  d.NA = d.NX + d.HP + 16;
  // Steps per weight-gradient chunk: as many as keep one dG chunk buffer within 64 MiB (the
  // staging is t-independent workspace), at least 2 and at most 32.  Every chunk costs one
  // read-modify-write of the whole dW accumulator, so longer chunks are cheaper per step.
  // Small batches get up to 64 steps (K = CH*B of at least 2048 where 64 MiB allow it): the dW
  // accumulator pass of a chunk otherwise outweighs its GEMM.
  const size_t step_bytes = (size_t)d.BP * d.G4 * (dtype ? 2 : 4);
  size_t ch = ((size_t)64 << 20) / step_bytes;
  d.CH = ch < 2 ? 2 : (ch > 32 ? 32 : (int)ch);
  if (d.CH == 32 && B <= 32 && ((size_t)64 << 20) / step_bytes >= 64) d.CH = 64;
  d.hplane = dtype ? (size_t)d.BP * d.KH : (size_t)B * H;
  d.unit = (d.hplane + (size_t)B * H + 63) / 64 * 64;
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

// Pointwise activations on the hardware exp2 / reciprocal units (a few ulp; the absolute error of
// tanh stays below 1e-7, far inside the fp32 gradient tolerance).
__device__ inline float sigmoidf_(float z) { return __frcp_rn(1.0f + __expf(-z)); }
__device__ inline float tanhf_(float z) {
  const float e = __expf(-2.0f * fabsf(z));            // in (0, 1]: no overflow
  return copysignf((1.0f - e) * __frcp_rn(1.0f + e), z);
}

// ---- the h plane of a hidden-state unit ----------------------------------------------------------
// (layout described in kernels.h).  HPlane<T>::store/load hide whether h is a plain fp32 plane or
// the split, fragment-tiled pair of 16-bit planes.
template <class T>
struct HPlane;

template <>
struct HPlane<float> {
  static constexpr bool SPLIT = false;
  __device__ static void store(float* plane, int b, int u, float v, int, int H, size_t) { plane[(size_t)b * H + u] = v; }
  __device__ static float load(const float* plane, int b, int u, int, int H, size_t) { return plane[(size_t)b * H + u]; }
  __device__ static float as_operand(const float* plane, int b, int u, int, int H, size_t) {
    return plane[(size_t)b * H + u];
  }
};

template <class T>
__device__ inline size_t ft_offset(int row, int k, int nsteps);

template <>
struct HPlane<__bf16> {
  static constexpr bool SPLIT = true;
  // nsh = KH / 32 macro steps per batch tile; half = BP * KH elements per 16-bit plane
  __device__ static void store(float* plane, int b, int u, float v, int nsh, int, size_t half) {
    unsigned short* hi = reinterpret_cast<unsigned short*>(plane);
    const unsigned bits = __float_as_uint(v);
    const size_t o = ft_offset<__bf16>(b, u, nsh);
    hi[o] = (unsigned short)((bits + 0x8000u) >> 16);
    hi[half + o] = (unsigned short)(bits & 0xffffu);
  }
  __device__ static float load(const float* plane, int b, int u, int nsh, int, size_t half) {
    const unsigned short* hi = reinterpret_cast<const unsigned short*>(plane);
    const size_t o = ft_offset<__bf16>(b, u, nsh);
    const unsigned lo = hi[half + o];
    return __uint_as_float((((unsigned)hi[o] - (lo >> 15)) << 16) | lo);
  }
  __device__ static __bf16 as_operand(const float* plane, int b, int u, int nsh, int, size_t) {
    const __bf16* hi = reinterpret_cast<const __bf16*>(plane);
    return hi[ft_offset<__bf16>(b, u, nsh)];
  }
};

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

// Operand arrays the library builds itself are stored "fragment-tiled": for a logical matrix
// M[rows][K] the element (row, k) lives at
//     (((row/16) * (K/KSTEP) + k/KSTEP) * 64 + ((k%KSTEP)/VEC)*16 + row%16) * VEC + k%VEC
// so that the 64 lanes of a wave fetch the fragment of one 16-row tile and one macro step as one
// contiguous, fully coalesced block of 64*VEC elements (1 KiB).
template <class T>
__device__ inline void ft_decode(size_t idx, int nsteps, int& row, int& k) {
  constexpr int VEC = Mma<T>::VEC, KSTEP = 4 * VEC;
  const int e = (int)(idx % VEC);
  const int lane = (int)((idx / VEC) % 64);
  const size_t blk = idx / (VEC * 64);
  const int kstep = (int)(blk % nsteps);
  const int tile = (int)(blk / nsteps);
  row = tile * 16 + (lane & 15);
  k = kstep * KSTEP + (lane >> 4) * VEC + e;
}

template <class T>
__device__ inline size_t ft_offset(int row, int k, int nsteps) {
  constexpr int VEC = Mma<T>::VEC, KSTEP = 4 * VEC;
  return ((((size_t)(row >> 4) * nsteps + k / KSTEP) * 64 + ((k % KSTEP) / VEC) * 16 + (row & 15)) * VEC) + k % VEC;
}

// The four packed rows 4u .. 4u+3 of hidden unit u, and which gate block of the caller's W_ih / W_hh
// feeds each of them (-1: that half of the row is zero).
//   LSTM: rows i, f, g, o, both halves from the same gate block.
//   GRU:  rows r, z, n_x, n_h.  The candidate's input part and recurrent part are kept as two rows
//         (n = tanh(n_x + r * n_h)), so one GEMM with the same 4-rows-per-unit shape serves both cells.
__host__ __device__ inline int packed_gate_x(int cell, int row) { return cell == 0 ? row : (row < 3 ? row : -1); }
__host__ __device__ inline int packed_gate_h(int cell, int row) { return cell == 0 ? row : (row == 2 ? -1 : (row == 3 ? 2 : row)); }

template <class T>
__global__ void prep_weights_kernel(Dims d, const float* __restrict__ W_ih, const float* __restrict__ W_hh,
                                    const float* __restrict__ b, T* __restrict__ Wp, float* __restrict__ bp,
                                    T* __restrict__ WTh, T* __restrict__ WTx) {
  constexpr int KSTEP = 4 * Mma<T>::VEC;
  const size_t nWp = (size_t)d.G4 * d.KP, nWTh = (size_t)d.HP * d.G4, nWTx = (size_t)d.NX * d.G4;
  const size_t total = nWp + nWTh + nWTx + (size_t)d.G4;
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
    if (idx < nWp) {   // Wp: logical [G4][KP], row' = 4u + gate
      int rowp, k;
      ft_decode<T>(idx, d.KP / KSTEP, rowp, k);
      int u = rowp >> 2, gate = rowp & 3;
      float v = 0.0f;
      if (u < d.H) {
        if (k < d.KX) {
          const int gx = packed_gate_x(d.cell, gate);
          if (k < d.I && gx >= 0) v = W_ih[((size_t)gx * d.H + u) * d.I + k];
        } else if (k - d.KX < d.H) {
          const int gh = packed_gate_h(d.cell, gate);
          if (gh >= 0) v = W_hh[((size_t)gh * d.H + u) * d.H + (k - d.KX)];
        }
      }
      Wp[idx] = (T)v;
    } else if (idx < nWp + nWTh + nWTx) {   // WTh: logical [HP][G4]; WTx: logical [NX][G4]; k' = 4u + gate
      size_t j = idx - nWp;
      bool is_h = j < nWTh;
      if (!is_h) j -= nWTh;
      int n, kp;
      ft_decode<T>(j, d.G4 / KSTEP, n, kp);
      int u = kp >> 2, gate = kp & 3;
      float v = 0.0f;
      if (u < d.H) {
        const int g = is_h ? packed_gate_h(d.cell, gate) : packed_gate_x(d.cell, gate);
        if (g >= 0) {
          const size_t row = (size_t)g * d.H + u;
          if (is_h) {
            if (n < d.H) v = W_hh[row * d.H + n];
          } else {
            if (n < d.I) v = W_ih[row * d.I + n];
          }
        }
      }
      (is_h ? WTh : WTx)[j] = (T)v;
    } else {
      int kp = (int)(idx - nWp - nWTh - nWTx);
      int u = kp >> 2, gate = kp & 3;
      float v = 0.0f;
      if (b != nullptr && u < d.H) {
        if (d.cell == 0) {
          v = b[(size_t)gate * d.H + u];
        } else {   // b = [b_ih (r, z, n) | b_hh (r, z, n)]
          const int gx = packed_gate_x(1, gate), gh = packed_gate_h(1, gate);
          if (gx >= 0) v += b[(size_t)gx * d.H + u];
          if (gh >= 0) v += b[(size_t)(3 + gh) * d.H + u];
        }
      }
      bp[kp] = v;
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

template <class T>
__global__ void init_state_kernel(Dims d, const float* __restrict__ h0, const float* __restrict__ c0,
                                  float* __restrict__ dst) {
  const int W = HPlane<T>::SPLIT ? d.KH : d.H;   // split layout: padding columns are written as zero
  const size_t n = (size_t)d.B * W;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride) {
    const int b = (int)(i / W), u = (int)(i % W);
    const size_t e = (size_t)b * d.H + u;
    HPlane<T>::store(dst, b, u, (u < d.H && h0) ? h0[e] : 0.0f, d.KH / 32, d.H, (size_t)d.BP * d.KH);
    if (u < d.H) dst[d.hplane + e] = c0 ? c0[e] : 0.0f;
  }
}

hipError_t launch_init_state(const Dims& d, const float* h0, const float* c0, float* dst_unit, hipStream_t st) {
  size_t n = (size_t)d.B * d.KH;
  size_t blocks = (n + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  if (d.dtype)
    init_state_kernel<__bf16><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(d, h0, c0, dst_unit);
  else
    init_state_kernel<float><<<dim3((unsigned)blocks), dim3(256), 0, st>>>(d, h0, c0, dst_unit);
  return hipGetLastError();
}

__global__ void copy_plane_kernel(size_t n, const float* __restrict__ src, float* __restrict__ dst, int accumulate) {
  size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < n; i += stride)
    dst[i] = accumulate == 2 ? 0.0f : (accumulate ? dst[i] + src[i] : src[i]);
}

hipError_t launch_copy_plane(const Dims& d, const float* src, float* dst, int accumulate, hipStream_t st) {
  size_t n = (size_t)d.B * d.H;
  size_t blocks = (n + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  copy_plane_kernel<<<dim3((unsigned)blocks), dim3(256), 0, st>>>(n, src, dst, accumulate);
  return hipGetLastError();
}

// ---- pointwise forward step of one (sequence, hidden unit) -------------------------------------
// G: the four gate-GEMM results of the unit (packed rows), bias: their biases, state_prev: c_{s-1}
// (LSTM) or h_{s-1} in full precision (GRU).  Returns h_s; `second` is what the second plane of
// the state unit keeps (LSTM: c_s; GRU: the recurrent part n_h of the candidate), `gate` the
// values the backward step needs (LSTM: i, f, g, o; GRU: r, z, n).  Every kernel that computes a
// forward step calls this one function, with the multiply-adds spelled out, so that a step gives
// the same bits whichever kernel ran it.
template <int CELL>
__device__ inline float cell_forward(const float (&G)[4], const float4& bias, float state_prev, float& second,
                                     float (&gate)[4]) {
  if (CELL == 0) {
    const float gi = sigmoidf_(G[0] + bias.x);
    const float gf = sigmoidf_(G[1] + bias.y);
    const float gg = tanhf_(G[2] + bias.z);
    const float go = sigmoidf_(G[3] + bias.w);
    const float c = __fmaf_rn(gf, state_prev, __fmul_rn(gi, gg));
    gate[0] = gi;
    gate[1] = gf;
    gate[2] = gg;
    gate[3] = go;
    second = c;
    return __fmul_rn(go, tanhf_(c));
  } else {
    // rows r, z, n_x, n_h: n = tanh(n_x + r * n_h), h = (1 - z) n + z h_prev
    const float r = sigmoidf_(G[0] + bias.x);
    const float z = sigmoidf_(G[1] + bias.y);
    const float nh = G[3] + bias.w;
    const float n = tanhf_(__fmaf_rn(r, nh, G[2] + bias.z));
    gate[0] = r;
    gate[1] = z;
    gate[2] = n;
    gate[3] = 0.0f;
    second = nh;
    return __fmaf_rn(1.0f - z, n, __fmul_rn(z, state_prev));
  }
}

// Pointwise backward step of one (sequence, hidden unit) of the LSTM: from dh_s (recurrent part
// plus injected loss gradient), the running dc, the internal state (i, f, g, o, c_s) and c_{s-1}
// to the four gate pre-activation gradients and dc_{s-1}.  One function, multiply-adds spelled
// out, for every kernel that runs a backward step: the same bits whichever kernel ran it.
__device__ inline void lstm_backward_point(float dh, float dc_in, float gi, float gf, float gg, float go, float c_s,
                                           float c_prev, float (&dG)[4], float& dc_out) {
  const float tc = tanhf_(c_s);
  const float d_o = __fmul_rn(dh, tc);
  const float dct = __fmaf_rn(__fmul_rn(dh, go), __fmaf_rn(-tc, tc, 1.0f), dc_in);
  dG[0] = __fmul_rn(__fmul_rn(__fmul_rn(dct, gg), gi), __fsub_rn(1.0f, gi));
  dG[1] = __fmul_rn(__fmul_rn(__fmul_rn(dct, c_prev), gf), __fsub_rn(1.0f, gf));
  dG[2] = __fmul_rn(__fmul_rn(dct, gi), __fmaf_rn(-gg, gg, 1.0f));
  dG[3] = __fmul_rn(__fmul_rn(d_o, go), __fsub_rn(1.0f, go));
  dc_out = __fmul_rn(dct, gf);
}

// The same for the GRU: r, z, n the gates, nh the recurrent part of the candidate (n = tanh(n_x + r * nh)),
// h_prev = h_{s-1} in full precision.  dh is the whole dL/dh_s: the GEMM part, the injected loss
// gradient and the part that bypasses the GEMM (dh_{s+1} * z_{s+1}, carried in the running plane).
// dG: gradients of the packed rows r, z, n_x, n_h; carry: what step s - 1 adds to its dh.
__device__ inline void gru_backward_point(float dh, float r, float z, float n, float nh, float h_prev, float (&dG)[4],
                                          float& carry) {
  const float da_n = __fmul_rn(__fmul_rn(dh, __fsub_rn(1.0f, z)), __fmaf_rn(-n, n, 1.0f));
  dG[0] = __fmul_rn(__fmul_rn(__fmul_rn(da_n, nh), r), __fsub_rn(1.0f, r));
  dG[1] = __fmul_rn(__fmul_rn(__fmul_rn(dh, __fsub_rn(h_prev, n)), z), __fsub_rn(1.0f, z));
  dG[2] = da_n;
  dG[3] = __fmul_rn(da_n, r);
  carry = __fmul_rn(dh, z);
}

// ---- forward step: gate GEMM + LSTM pointwise -------------------------------------------------

struct FwdParams {
  const void* Wp;
  const float* bp;
  const float* x_s;
  const float* src_h;   // h plane of the input state (layout: HPlane)
  const float* src_c;
  float* dst_h;         // h plane of the output state
  float* dst_c;
  float* g_i;   // NULL: do not keep the gates
  float* g_f;
  float* g_g;
  float* g_o;
  int B, I, H, HP, KX, KH, KP, BP;
};

// Raw (unconverted) activation fragment: VEC fp32 values, zero beyond `limit`.
template <int VEC>
struct RawAct {
  float v[VEC];
};
template <int VEC>
__device__ inline RawAct<VEC> load_raw(const float* __restrict__ row, int k, int limit, bool vec_ok) {
  RawAct<VEC> r;
  if (vec_ok && k + VEC <= limit) {
#pragma unroll
    for (int e = 0; e < VEC; e += 4) {
      float4 q = *reinterpret_cast<const float4*>(row + k + e);
      r.v[e] = q.x;
      r.v[e + 1] = q.y;
      r.v[e + 2] = q.z;
      r.v[e + 3] = q.w;
    }
  } else {
#pragma unroll
    for (int e = 0; e < VEC; ++e) r.v[e] = (k + e < limit) ? row[k + e] : 0.0f;
  }
  return r;
}

// As load_raw for rows whose length is a multiple of VEC (k is one too): a fragment lies wholly
// inside the row or wholly outside, so one address clamp and one select replace the branches.
// (Branches that load into the same registers make the compiler wait for every outstanding memory
// operation between them.)
template <int VEC>
__device__ inline RawAct<VEC> load_raw_whole(const float* __restrict__ row, int k, int limit) {
  RawAct<VEC> r;
  const bool inside = k < limit;
  const float* src = row + (inside ? k : 0);
#pragma unroll
  for (int e = 0; e < VEC; e += 4) {
    const float4 q = *reinterpret_cast<const float4*>(src + e);
    r.v[e] = inside ? q.x : 0.0f;
    r.v[e + 1] = inside ? q.y : 0.0f;
    r.v[e + 2] = inside ? q.z : 0.0f;
    r.v[e + 3] = inside ? q.w : 0.0f;
  }
  return r;
}

// One workgroup of 64*KS threads = BT batch tiles (16 sequences each) x NG unit groups (4 hidden
// units = 16 gate rows each).  Its KS waves split the K axis; every wave covers all NG x BT output
// tiles (each weight fragment is reused for BT batch tiles, each activation fragment for NG unit
// groups) and issues all loads of U macro steps before the first MFMA, so that several KiB per
// wave are in flight.  Partial sums meet in LDS (`red`, forward_red_floats(NG, BT, KS) floats) and
// are added in a fixed order by the thread that then does the LSTM pointwise step of that
// (sequence, unit).  (bx, by) = (unit-group tile, batch-tile group).
template <class T, int NG, int BT, int KS, int U, int CELL>
__device__ inline void forward_body(const FwdParams& p, int bx, int by, float* red) {
  using M = Mma<T>;
  constexpr int VEC = M::VEC, KSTEP = 4 * VEC;
  // wave_index note: the wave index is read into a scalar register.  Conditions on it then compile
  // to scalar branches; as a vector value they become lane masks, and an MFMA under a lane mask that
  // is empty still executes (short masked blocks get no branch around them).
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), lane = threadIdx.x & 63;   // scalar: see wave_index note
  if (wave >= KS) return;   // surplus waves of a wider (fused) workgroup leave before any barrier
  const int lrow = lane & 15, lq = lane >> 4;
  const int group0 = bx * NG;
  const int ngroups = p.HP >> 2;
  const int b0 = by * BT * 16;
  using HP_ = HPlane<T>;
  const bool x_vec = (p.I & 3) == 0, h_vec = (p.H & 3) == 0;
  const int nsteps = p.KP / KSTEP;
  const int nsx = p.KX / KSTEP, nsh = p.KH / KSTEP;   // macro steps of the x and the h segment
  const size_t hhalf = (size_t)p.BP * p.KH;           // elements of one 16-bit plane (split layout)
  const float* xrow[BT];
  const float* hrow[BT];   // plain layout: row pointer
  const T* hfrag[BT];      // split layout: this lane's slot in the batch tile's first fragment
#pragma unroll
  for (int t = 0; t < BT; ++t) {
    const int b_ld = min(b0 + t * 16 + lrow, p.B - 1);
    xrow[t] = p.x_s + (size_t)b_ld * p.I;
    hrow[t] = p.src_h + (size_t)b_ld * p.H;
    const int btile = min(by * BT + t, p.BP / 16 - 1);
    hfrag[t] = reinterpret_cast<const T*>(p.src_h) + ((size_t)btile * nsh * 64 + lane) * VEC;
  }
  const T* wbase[NG];   // fragment-tiled: tile (group) stride = nsteps * 64 * VEC
#pragma unroll
  for (int g = 0; g < NG; ++g) {
    int grp = min(group0 + g, ngroups - 1);
    wbase[g] = reinterpret_cast<const T*>(p.Wp) + ((size_t)grp * nsteps * 64 + lane) * VEC;
  }
  f32x4 acc[NG][BT];
#pragma unroll
  for (int g = 0; g < NG; ++g)
#pragma unroll
    for (int t = 0; t < BT; ++t) acc[g][t] = f32x4{0.f, 0.f, 0.f, 0.f};

  // Epilogue work is dealt out by memory layout, not by MFMA layout: item i of the workgroup's
  // BT*16 rows x UW units is (row, unit) with the unit index fastest, so that consecutive lanes
  // own consecutive units of one sequence and every pointwise load and store of a wave falls
  // into runs of UW*4 bytes (plain planes) or 16 bytes (the 16-bit h planes) instead of one
  // element per row.  The operands are fetched now, so that their latency hides behind the K loop.
  constexpr int UW = NG * 4, RS = UW + 1;          // units per workgroup; padded row stride in `red`
  constexpr int ITEMS = BT * 16 * UW, NTHR = 64 * KS, IPT = (ITEMS + NTHR - 1) / NTHR;
  bool epi[IPT];
  size_t eidx[IPT];
  int eb[IPT], eu[IPT];
  float4 bias[IPT];
  float c_prev[IPT];
#pragma unroll
  for (int q = 0; q < IPT; ++q) {
    const int item = (int)threadIdx.x + q * NTHR;
    const int b = b0 + (item / UW) % (BT * 16);     // rows of batch tile t follow those of t-1
    const int u = group0 * 4 + item % UW;
    epi[q] = item < ITEMS && b < p.B && u < p.H;
    eidx[q] = (size_t)b * p.H + u;
    eb[q] = item < ITEMS ? b : p.B;
    eu[q] = u;
    bias[q] = float4{0.f, 0.f, 0.f, 0.f};
    c_prev[q] = 0.0f;
    if (epi[q]) {
      bias[q] = *reinterpret_cast<const float4*>(p.bp + 4 * u);
      // the state the pointwise step blends with: c_{s-1} (LSTM) or h_{s-1} in full precision (GRU)
      c_prev[q] = CELL ? HP_::load(p.src_h, b, u, nsh, p.H, hhalf) : p.src_c[eidx[q]];
    }
  }

  // This wave's macro steps wave, wave + KS, ... in rising order: first those of the x segment
  // (and, in the plain layout, all of them), U at a time: all loads, then all MFMAs.  When every
  // row length is a multiple of the fragment width the loads are the branch-free ones (a loader
  // with branches makes the compiler wait for all outstanding loads between fragments); the
  // choice is made once, outside the loop.
  const int n_batch = HP_::SPLIT ? nsx : nsteps;   // macro steps handled by the batched loop
  auto batched = [&](auto whole_tag) {
    constexpr bool WHOLE = decltype(whole_tag)::value;
    for (int s0 = wave; s0 < n_batch; s0 += KS * U) {
      RawAct<VEC> rb[U][BT];          // fp32 activations still to be converted (x; h in the plain layout)
      typename M::Frag af[U][NG];
#pragma unroll
      for (int uu = 0; uu < U; ++uu) {
        const int s = min(s0 + uu * KS, n_batch - 1);   // clamped: the surplus fragment is discarded
        const int k = s * KSTEP + VEC * lq;
#pragma unroll
        for (int t = 0; t < BT; ++t) {
          if (WHOLE)
            rb[uu][t] = s < nsx ? load_raw_whole<VEC>(xrow[t], k, p.I) : load_raw_whole<VEC>(hrow[t], k - p.KX, p.H);
          else if (s < nsx)
            rb[uu][t] = load_raw<VEC>(xrow[t], k, p.I, x_vec);
          else
            rb[uu][t] = load_raw<VEC>(hrow[t], k - p.KX, p.H, h_vec);
        }
#pragma unroll
        for (int g = 0; g < NG; ++g) af[uu][g] = M::load(wbase[g] + (size_t)s * 64 * VEC);
      }
#pragma unroll
      for (int uu = 0; uu < U; ++uu) {
        const int s = s0 + uu * KS;
        if (s < n_batch) {
#pragma unroll
          for (int t = 0; t < BT; ++t) {
            typename M::Frag bf = M::from_f32(rb[uu][t].v);
#pragma unroll
            for (int g = 0; g < NG; ++g) acc[g][t] = M::mma(af[uu][g], bf, acc[g][t]);
          }
        }
      }
    }
  };
  if (p.I % VEC == 0 && (HP_::SPLIT || p.H % VEC == 0))
    batched(std::true_type{});
  else
    batched(std::false_type{});
  if (HP_::SPLIT) {
    // The h segment (ready-made fragments: every load is 16 bytes per lane, no branches) runs
    // through a ring of U register slots: a slot is refilled with the step U ahead as soon as its
    // MFMAs are issued, so U steps' loads stay in flight while the matrix pipe works, instead of
    // the pipe idling through every batch of loads.  The main loop has no conditions (the compiler
    // can then wait for exactly the loads a step needs); the last steps are peeled.
    const int sh0 = wave >= nsx ? wave : wave + KS * ((nsx - wave + KS - 1) / KS);   // this wave's first h step
    typename M::Frag af[U][NG], hb[U][BT];
    auto load_slot = [&](int u, int step) {
      const int sc = min(step, nsteps - 1);   // clamped: a surplus fragment is discarded
#pragma unroll
      for (int t = 0; t < BT; ++t) hb[u][t] = M::load(hfrag[t] + (size_t)(sc - nsx) * 64 * VEC);
#pragma unroll
      for (int g = 0; g < NG; ++g) af[u][g] = M::load(wbase[g] + (size_t)sc * 64 * VEC);
    };
    auto mma_slot = [&](int u) {
#pragma unroll
      for (int t = 0; t < BT; ++t)
#pragma unroll
        for (int g = 0; g < NG; ++g) acc[g][t] = M::mma(af[u][g], hb[u][t], acc[g][t]);
    };
    if (sh0 < nsteps) {
#pragma unroll
      for (int u = 0; u < U; ++u) load_slot(u, sh0 + u * KS);
      int s = sh0;
      for (; s + KS * (2 * U - 1) < nsteps; s += KS * U) {   // every refill target is a real step
#pragma unroll
        for (int u = 0; u < U; ++u) {
          mma_slot(u);
          load_slot(u, s + (u + U) * KS);
        }
      }
      // what the slots hold now, then at most U - 1 further steps, fetched as a batch
#pragma unroll
      for (int u = 0; u < U; ++u)
        if (s + u * KS < nsteps) mma_slot(u);
      s += KS * U;
      if (s < nsteps) {
#pragma unroll
        for (int u = 0; u < U; ++u) load_slot(u, s + u * KS);
#pragma unroll
        for (int u = 0; u < U; ++u)
          if (s + u * KS < nsteps) mma_slot(u);
      }
    }
  }

  // partial sums -> red[wave][gate r][row][unit] (row stride padded against bank conflicts)
#pragma unroll
  for (int g = 0; g < NG; ++g)
#pragma unroll
    for (int t = 0; t < BT; ++t)
#pragma unroll
      for (int r = 0; r < 4; ++r) red[((wave * 4 + r) * BT * 16 + t * 16 + lrow) * RS + g * 4 + lq] = acc[g][t][r];
  __syncthreads();
#pragma unroll
  for (int q = 0; q < IPT; ++q) {
    const int item = (int)threadIdx.x + q * NTHR;
    if (item >= ITEMS) break;
    const int cell = ((item / UW) % (BT * 16)) * RS + item % UW;
    float G[4] = {0.f, 0.f, 0.f, 0.f};
    for (int w = 0; w < KS; ++w)   // fixed order: results do not depend on scheduling
#pragma unroll
      for (int r = 0; r < 4; ++r) G[r] += red[(w * 4 + r) * BT * 16 * RS + cell];
    if (!epi[q]) {
      // split layout: the padding columns H..KH of a valid row are part of the operand other
      // launches fetch, so they are (re)written as zero with every state
      if (HP_::SPLIT && eb[q] < p.B && eu[q] < p.KH) HP_::store(p.dst_h, eb[q], eu[q], 0.0f, nsh, p.H, hhalf);
      continue;
    }
    const size_t e = eidx[q];
    float second, gate[4];
    const float h = cell_forward<CELL>(G, bias[q], c_prev[q], second, gate);
    HP_::store(p.dst_h, eb[q], eu[q], h, nsh, p.H, hhalf);
    p.dst_c[e] = second;
    if (p.g_i) {
      p.g_i[e] = gate[0];
      p.g_f[e] = gate[1];
      p.g_g[e] = gate[2];
      if (CELL == 0) p.g_o[e] = gate[3];
    }
  }
}

// Floats of LDS a forward workgroup needs for its partial sums.
constexpr int forward_red_floats(int NG, int BT, int KS) { return KS * 4 * BT * 16 * (NG * 4 + 1); }

template <class T, int NG, int BT, int KS, int U, int CELL>
__global__ __launch_bounds__(64 * KS) void forward_kernel(FwdParams p) {
  __shared__ float red[forward_red_floats(NG, BT, KS)];
  forward_body<T, NG, BT, KS, U, CELL>(p, blockIdx.x, blockIdx.y, red);
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
  int B, H, HP, KH, G4, NX, KC, BP;
  int cell;     // 0 LSTM, 1 GRU
};

// One workgroup of 64*KS threads = NT hidden-unit tiles x BT batch tiles (16 x 16 outputs each);
// its KS waves split K = 4*HP, every wave covering all NT x BT tiles and issuing the loads of U
// macro steps before the first MFMA.  Partial sums meet in LDS (`red`, KS*NT*BT*256 floats).  The
// pointwise backward has NT*BT*4 pieces of work (tile x which of the lane's four hidden units),
// dealt round-robin to the waves.  (bx, by) = (hidden-unit tile group, batch-tile group).
template <class T, int NT, int BT, int KS, int U>
__device__ inline void backward_body(const BwdParams& p, int bx, int by, float* red) {
  using M = Mma<T>;
  constexpr int VEC = M::VEC, KSTEP = 4 * VEC;
  constexpr int NTILE = NT * BT, NPIECE = NTILE * 4, PPW = (NPIECE + KS - 1) / KS;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), lane = threadIdx.x & 63;   // scalar: see wave_index note
  if (wave >= KS) return;   // surplus waves of a wider (fused) workgroup leave before any barrier
  const int lrow = lane & 15, lq = lane >> 4;
  const int ntiles_n = p.HP / 16, ntiles_b = p.BP / 16;
  // Epilogue pieces of this wave: piece id = tile * 4 + r, tile = tn * BT + tb.  Their pointwise
  // operands are fetched before the K loop so that the latency overlaps with it.
  bool epi[PPW];
  size_t eidx[PPW];
  int en[PPW], eb[PPW];
  float h[PPW], dy[PPW], gi[PPW], gf[PPW], gg[PPW], go[PPW], c_s[PPW], c_prev[PPW], dc_in[PPW], h_prev[PPW];
#pragma unroll
  for (int q = 0; q < PPW; ++q) {
    const int piece = wave + q * KS;
    const int tile = piece >> 2, r = piece & 3;
    const int tn = tile / BT, tb = tile % BT;
    const int b = (by * BT + tb) * 16 + lrow;
    const int n = (bx * NT + tn) * 16 + 4 * lq + r;
    epi[q] = piece < NPIECE && b < p.B && n < p.H;
    eidx[q] = (size_t)b * p.H + n;
    en[q] = n;
    eb[q] = b;
    h[q] = dy[q] = gi[q] = gf[q] = gg[q] = go[q] = c_s[q] = c_prev[q] = dc_in[q] = h_prev[q] = 0.f;
    if (epi[q]) {
      const size_t e = eidx[q];
      if (p.dy_is_h || p.y_out_s) h[q] = HPlane<T>::load(p.h, b, n, p.KH / 32, p.H, (size_t)p.BP * p.KH);
      if (!p.dy_is_h && p.dy_s) dy[q] = p.dy_s[e];
      gi[q] = p.g_i[e];
      gf[q] = p.g_f[e];
      gg[q] = p.g_g[e];
      c_s[q] = p.c[e];
      dc_in[q] = p.dc[e];
      h_prev[q] = (float)HPlane<T>::as_operand(p.h_prev, b, n, p.KH / 32, p.H, (size_t)p.BP * p.KH);
      if (p.cell == 0) {
        go[q] = p.g_o[e];
        c_prev[q] = p.c_prev[e];
      } else {   // GRU blends with h_{s-1} itself: its full-precision value takes c_prev's place
        c_prev[q] = HPlane<T>::load(p.h_prev, b, n, p.KH / 32, p.H, (size_t)p.BP * p.KH);
      }
    }
  }
  if (p.dG_next) {
    f32x4 acc[NT][BT];
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
      for (int j = 0; j < BT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
    const int nsteps = p.G4 / KSTEP;
    const T* abase[NT];
    const T* bbase[BT];
#pragma unroll
    for (int i = 0; i < NT; ++i)
      abase[i] = reinterpret_cast<const T*>(p.WTh) + ((size_t)min(bx * NT + i, ntiles_n - 1) * nsteps * 64 + lane) * VEC;
#pragma unroll
    for (int j = 0; j < BT; ++j)
      bbase[j] = reinterpret_cast<const T*>(p.dG_next) + ((size_t)min(by * BT + j, ntiles_b - 1) * nsteps * 64 + lane) * VEC;
    // This wave's macro steps are wave, wave + KS, ...: nw of them.  A ring of U fragment slots
    // keeps U steps in flight from the first load to the last: slot u is refilled with the step U
    // places further on as soon as its MFMAs are issued.  Steps are consumed in the same order
    // as a plain loop would, so the sums are unchanged.  The main loop covers whole groups of U
    // steps that all have a refill, so its body has no branches and the number of loads
    // outstanding at every wait is known at compile time; the tail (at most two groups) is
    // conditional.
    const int nw = (nsteps - wave + KS - 1) / KS;
    typename M::Frag af[U][NT], bf[U][BT];
    auto load_slot = [&](int u, int j) {   // j: index into this wave's steps (always < nw here or clamped)
      const size_t off = (size_t)min(wave + j * KS, nsteps - 1) * 64 * VEC;
#pragma unroll
      for (int i = 0; i < NT; ++i) af[u][i] = M::load(abase[i] + off);
#pragma unroll
      for (int jj = 0; jj < BT; ++jj) bf[u][jj] = M::load(bbase[jj] + off);
    };
    auto mma_slot = [&](int u) {
#pragma unroll
      for (int i = 0; i < NT; ++i)
#pragma unroll
        for (int jj = 0; jj < BT; ++jj) acc[i][jj] = M::mma(af[u][i], bf[u][jj], acc[i][jj]);
    };
#pragma unroll
    for (int u = 0; u < U; ++u) load_slot(u, u);   // surplus slots (u >= nw) hold a clamped copy and are never used
    int j0 = 0;
    for (; j0 + 2 * U <= nw; j0 += U) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        mma_slot(u);
        load_slot(u, j0 + u + U);
      }
    }
    for (; j0 < nw; j0 += U) {
#pragma unroll
      for (int u = 0; u < U; ++u) {
        if (j0 + u < nw) mma_slot(u);
        if (j0 + u + U < nw) load_slot(u, j0 + u + U);
      }
    }
#pragma unroll
    for (int i = 0; i < NT; ++i)
#pragma unroll
      for (int j = 0; j < BT; ++j)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[((wave * NTILE + i * BT + j) * 4 + r) * 64 + lane] = acc[i][j][r];
    __syncthreads();
  }
#pragma unroll
  for (int q = 0; q < PPW; ++q) {
    const int piece = wave + q * KS;
    if (piece >= NPIECE) break;
    float dh = 0.0f;
    if (p.dG_next)
      for (int w = 0; w < KS; ++w) dh += red[(w * NPIECE + piece) * 64 + lane];   // fixed order
    if (!epi[q]) continue;
    const size_t e = eidx[q];
    const int n = en[q], b = eb[q];
    dh += p.dy_is_h ? h[q] : dy[q];
    if (p.y_out_s) p.y_out_s[e] = h[q];
    float dGi, dGf, dGg, dGo;
    if (p.cell == 0) {
      float dG[4], dc_out;
      lstm_backward_point(dh, dc_in[q], gi[q], gf[q], gg[q], go[q], c_s[q], c_prev[q], dG, dc_out);
      dGi = dG[0];
      dGf = dG[1];
      dGg = dG[2];
      dGo = dG[3];
      p.dc[e] = dc_out;
    } else {
      // GRU: r = gi, z = gf, n = gg, n_h = c_s, h_{s-1} = c_prev.  The running plane `dc` carries
      // the part of dL/dh_{s-1} that bypasses the GEMM: dh_s * z_s.
      float dG[4], carry;
      gru_backward_point(__fadd_rn(dh, dc_in[q]), gi[q], gf[q], gg[q], c_s[q], c_prev[q], dG, carry);
      dGi = dG[0];
      dGf = dG[1];
      dGg = dG[2];
      dGo = dG[3];
      p.dc[e] = carry;
    }
    const T q0 = (T)dGi, q1 = (T)dGf, q2 = (T)dGg, q3 = (T)dGo;
    // dG of this step, fragment-tiled [b][4n + gate]: the four gates are consecutive in one lane slot
    T* dG4 = reinterpret_cast<T*>(p.dG_cur) + ft_offset<T>(b, 4 * n, p.G4 / KSTEP);
    dG4[0] = q0;
    dG4[1] = q1;
    dG4[2] = q2;
    dG4[3] = q3;
    // transposed copies for the weight gradient, fragment-tiled [4n + gate][col] and [NX + n][col]
    const int col = p.col0 + b, ncs = p.KC / KSTEP;
    T* dGT = reinterpret_cast<T*>(p.dGT);
    dGT[ft_offset<T>(4 * n + 0, col, ncs)] = q0;
    dGT[ft_offset<T>(4 * n + 1, col, ncs)] = q1;
    dGT[ft_offset<T>(4 * n + 2, col, ncs)] = q2;
    dGT[ft_offset<T>(4 * n + 3, col, ncs)] = q3;
    reinterpret_cast<T*>(p.aT)[ft_offset<T>(p.NX + n, col, ncs)] = (T)h_prev[q];
  }
}

template <class T, int NT, int BT, int KS, int U>
__global__ __launch_bounds__(64 * KS) void backward_kernel(BwdParams p) {
  __shared__ float red[KS * NT * BT * 4 * 64];
  backward_body<T, NT, BT, KS, U>(p, blockIdx.x, blockIdx.y, red);
}

// ---- fused launch: a backward step and an independent forward step ---------------------------
// The recomputation chain (forward operations) never depends on the backward chain, so the
// forward operation that follows a backward step in the schedule can share its launch whenever
// it does not overwrite a state that backward step still reads.  Workgroups [0, nf) play the
// forward role, the rest the backward role; 512 threads each, and the launch bounds hold the kernel
// to 128 registers (4 waves per SIMD), so that two workgroups are resident on a compute unit at
// the same time and the 2 x 256 workgroups of a launch run as one wave of work, not two.  Each role splits K over the
// same number of waves as its stand-alone kernel, so sums are formed in the same order and results
// do not depend on whether a step was fused.
constexpr int PAIR_FKS = 8, PAIR_NG = 4, PAIR_FU = 1, PAIR_BKS = 8, PAIR_BU = 4;

// Roles of one fused launch: forward tile FNG x 1 split over FKS waves, backward tile BNT x BBT over
// BKS waves (the K splits of the stand-alone kernels of the same shape class).  FU and BU, the
// macro steps a wave keeps in flight, are smaller than the stand-alone kernels': two resident
// workgroups share a compute unit's load path, and measured launch times fall as the queues get
// shorter (large-K class: 9.98 us at FU, BU = 2, 8; 9.47 us at 1, 4; small-K class 12.2 -> 10.8 us).
template <class T, int CELL, int FNG, int FKS, int FU, int BNT, int BBT, int BKS, int BU>
__global__ __launch_bounds__(64 * (FKS > BKS ? FKS : BKS), 4) void pair_kernel(FwdParams f, BwdParams b, int nfx, int nf,
                                                                             int nbx) {
  constexpr int FRED = forward_red_floats(FNG, 1, FKS), BRED = BKS * BNT * BBT * 4 * 64;
  __shared__ float red[FRED > BRED ? FRED : BRED];
  const int id = blockIdx.x;
  if (id < nf)
    forward_body<T, FNG, 1, FKS, FU, CELL>(f, id % nfx, id / nfx, red);
  else
    backward_body<T, BNT, BBT, BKS, BU>(b, (id - nf) % nbx, (id - nf) / nbx, red);
}

// Kernel configurations by shape.  Tiles per workgroup grow with the problem so that the grid
// stays near one workgroup per compute unit while every operand byte is reused as often as
// possible; the choice depends on the shape only, never on the schedule.
enum FwdConfig { FWD_TINY, FWD_SMALLK, FWD_B1, FWD_42, FWD_82 };
enum BwdConfig { BWD_SMALLK, BWD_11, BWD_12, BWD_22 };
constexpr int TARGET_WGS = 256;

template <class T>
static FwdConfig forward_config(const Dims& d) {
  const int nsteps = d.KP / (4 * Mma<T>::VEC);
  if (nsteps <= 8) return FWD_TINY;
  if (nsteps <= 20) return FWD_SMALLK;
  const int ngroups = d.HP / 4, bt = d.BP / 16;
  if (bt >= 2 && ((ngroups + 7) / 8) * ((bt + 1) / 2) >= TARGET_WGS) return FWD_82;
  if (bt >= 2 && ((ngroups + 3) / 4) * ((bt + 1) / 2) >= TARGET_WGS) return FWD_42;
  return FWD_B1;
}

template <class T>
static BwdConfig backward_config(const Dims& d) {
  const int nsteps = d.G4 / (4 * Mma<T>::VEC);
  if (nsteps <= 16) return BWD_SMALLK;
  const int nt = d.HP / 16, bt = d.BP / 16;
  if (nt >= 2 && bt >= 2 && ((nt + 1) / 2) * ((bt + 1) / 2) >= TARGET_WGS) return BWD_22;
  if (bt >= 2 && nt * ((bt + 1) / 2) >= TARGET_WGS) return BWD_12;
  return BWD_11;
}

template <class T, int NG, int BT, int KS, int U>
static hipError_t launch_forward_cfg(const Dims& d, const FwdParams& p, hipStream_t st) {
  dim3 grid((d.HP / 4 + NG - 1) / NG, (d.BP / 16 + BT - 1) / BT), block(64 * KS);
  if (d.cell)
    forward_kernel<T, NG, BT, KS, U, 1><<<grid, block, 0, st>>>(p);
  else
    forward_kernel<T, NG, BT, KS, U, 0><<<grid, block, 0, st>>>(p);
  return hipGetLastError();
}

template <class T>
static hipError_t launch_forward_t(const Dims& d, const FwdParams& p, hipStream_t st) {
  switch (forward_config<T>(d)) {
    case FWD_TINY: return launch_forward_cfg<T, 1, 1, 4, 2>(d, p, st);   // tiny K: one small workgroup per tile
    case FWD_SMALLK: return launch_forward_cfg<T, 4, 1, 4, 5>(d, p, st);
    case FWD_82: return launch_forward_cfg<T, 8, 2, 8, 1>(d, p, st);
    case FWD_42: return launch_forward_cfg<T, 4, 2, 8, 3>(d, p, st);
    default: return launch_forward_cfg<T, PAIR_NG, 1, PAIR_FKS, 5>(d, p, st);
  }
}

static FwdParams make_fwd_params(const Dims& d, const void* Wp, const float* bp, const float* x_s,
                                 const float* src_unit, float* dst_unit, float* gates_units) {
  const size_t plane = (size_t)d.B * d.H;
  FwdParams p{};
  p.Wp = Wp;
  p.bp = bp;
  p.x_s = x_s;
  p.src_h = src_unit;
  p.src_c = src_unit + d.hplane;
  p.dst_h = dst_unit;
  p.dst_c = dst_unit + d.hplane;
  if (gates_units) {   // two units: (i, f) and (g, o)
    p.g_i = gates_units;
    p.g_f = gates_units + plane;
    p.g_g = gates_units + d.unit;
    p.g_o = gates_units + d.unit + plane;
  }
  p.B = d.B;
  p.I = d.I;
  p.H = d.H;
  p.HP = d.HP;
  p.KX = d.KX;
  p.KH = d.KH;
  p.KP = d.KP;
  p.BP = d.BP;
  return p;
}

hipError_t launch_forward(const Dims& d, const void* Wp, const float* bp, const float* x_s, const float* src_unit,
                          float* dst_unit, float* gates_units, hipStream_t st) {
  FwdParams p = make_fwd_params(d, Wp, bp, x_s, src_unit, dst_unit, gates_units);
  return d.dtype ? launch_forward_t<__bf16>(d, p, st) : launch_forward_t<float>(d, p, st);
}

// ---- independent forward operations in one launch ----------------------------------------------
// Where every step of a stretch has its input hidden state in memory, the forward operations that
// recompute the steps' internal states do not depend on each other: they go out as one launch,
// grid.z = the operation.  A workgroup is a forward workgroup of its step (forward_body, with the K
// split of the shape's stand-alone kernel, so a step gives the same bits whichever launch ran it).
constexpr int FWD_BATCH_MAX_STEPS = 32;
struct FwdBatchSteps {
  const float* x[FWD_BATCH_MAX_STEPS];     // x_s [B, I]
  const float* src[FWD_BATCH_MAX_STEPS];   // unit (h_{s-1}, c_{s-1})
  float* dst[FWD_BATCH_MAX_STEPS];         // three units: (h_s, c_s), (i, f), (g, o)
};

template <class T, int NG, int BT, int KS, int U, int CELL>
__global__ __launch_bounds__(64 * KS) void forward_batch_kernel(FwdParams p, FwdBatchSteps steps, size_t hplane, size_t unit,
                                                                size_t plane) {
  __shared__ float red[forward_red_floats(NG, BT, KS)];
  const int j = blockIdx.z;
  float* dst = steps.dst[j];
  p.x_s = steps.x[j];
  p.src_h = steps.src[j];
  p.src_c = steps.src[j] + hplane;
  p.dst_h = dst;
  p.dst_c = dst + hplane;
  p.g_i = dst + unit;
  p.g_f = dst + unit + plane;
  p.g_g = dst + 2 * unit;
  p.g_o = dst + 2 * unit + plane;
  forward_body<T, NG, BT, KS, U, CELL>(p, blockIdx.x, blockIdx.y, red);
}

int forward_batch_max_steps() { return FWD_BATCH_MAX_STEPS; }
bool can_run_forward_batch(const Dims& d) { return d.dtype == 1; }

hipError_t launch_forward_batch(const Dims& d, const void* Wp, const float* bp, int n, const float* const* x,
                                const float* const* src, float* const* dst, hipStream_t st) {
  if (!can_run_forward_batch(d) || n < 1 || n > FWD_BATCH_MAX_STEPS) return hipErrorInvalidValue;
  FwdParams p = make_fwd_params(d, Wp, bp, x[0], src[0], dst[0], dst[0] + d.unit);
  FwdBatchSteps steps{};
  for (int j = 0; j < n; ++j) {
    steps.x[j] = x[j];
    steps.src[j] = src[j];
    steps.dst[j] = dst[j];
  }
  // 64 gate rows x 32 sequences per workgroup, two macro steps in flight per wave: two workgroups
  // fit a compute unit.  Measured on H = 1024, B = 64: 2.7 us per operation; 64 x 64 tiles 3.1 us,
  // three or four macro steps in flight 4.4 - 5.1 us.
  constexpr int NG = 4, BT = 2, FU = 2;
  const dim3 grid((d.HP / 4 + NG - 1) / NG, (d.BP / 16 + BT - 1) / BT, n);
  const size_t plane = (size_t)d.B * d.H;
  const FwdConfig cfg = forward_config<__bf16>(d);
  const bool small_k = cfg == FWD_TINY || cfg == FWD_SMALLK;   // the K split of the shape's stand-alone forward kernel
  if (small_k && d.cell)
    forward_batch_kernel<__bf16, NG, BT, 4, FU, 1><<<grid, dim3(64 * 4), 0, st>>>(p, steps, d.hplane, d.unit, plane);
  else if (small_k)
    forward_batch_kernel<__bf16, NG, BT, 4, FU, 0><<<grid, dim3(64 * 4), 0, st>>>(p, steps, d.hplane, d.unit, plane);
  else if (d.cell)
    forward_batch_kernel<__bf16, NG, BT, 8, FU, 1><<<grid, dim3(64 * 8), 0, st>>>(p, steps, d.hplane, d.unit, plane);
  else
    forward_batch_kernel<__bf16, NG, BT, 8, FU, 0><<<grid, dim3(64 * 8), 0, st>>>(p, steps, d.hplane, d.unit, plane);
  return hipGetLastError();
}

// ---- measurement: the bytes of a forward launch, streamed -----------------------------------
// The grid and block of the forward launch of this shape; every workgroup reads the weight panel
// (its gate rows x K, GEMM operand type) and the activation panel (its sequences x K: x in fp32, h
// in the operand type) its forward counterpart reads, from the same weight array, with the same
// 16-byte-per-lane loads, eight in flight per wave -- and does nothing else.  What this takes is
// what the memory system needs to deliver the launch's bytes to the compute units.
__global__ __launch_bounds__(512) void stream_panels_kernel(const uint4* __restrict__ w, size_t w_panel, const uint4* __restrict__ a,
                                                            size_t a_panel, float* __restrict__ sink) {
  constexpr int U = 8;
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), lane = threadIdx.x & 63, nwaves = blockDim.x >> 6;
  float acc = 0.0f;
  for (int part = 0; part < 2; ++part) {
    const uint4* base = part ? a + (size_t)blockIdx.y * a_panel : w + (size_t)blockIdx.x * w_panel;
    const size_t nblk = (part ? a_panel : w_panel) / 64;   // blocks of 64 x 16 bytes
    for (size_t b0 = wave; b0 < nblk; b0 += (size_t)nwaves * U) {
      uint4 v[U];
#pragma unroll
      for (int u = 0; u < U; ++u) {
        size_t b = b0 + (size_t)u * nwaves;
        if (b >= nblk) b = nblk - 1;
        v[u] = base[b * 64 + lane];
      }
#pragma unroll
      for (int u = 0; u < U; ++u) acc += __uint_as_float(v[u].x ^ v[u].y ^ v[u].z ^ v[u].w);
    }
  }
  if (acc == 12345.678f) sink[0] = acc;   // keeps the loads alive; never true in practice
}

template <class T>
static void forward_launch_shape(const Dims& d, int& ng, int& bt, int& ks) {
  switch (forward_config<T>(d)) {
    case FWD_TINY: ng = 1, bt = 1, ks = 4; break;
    case FWD_SMALLK: ng = 4, bt = 1, ks = 4; break;
    case FWD_82: ng = 8, bt = 2, ks = 8; break;
    case FWD_42: ng = 4, bt = 2, ks = 8; break;
    default: ng = PAIR_NG, bt = 1, ks = PAIR_FKS; break;
  }
}

hipError_t launch_forward_stream(const Dims& d, const void* Wp, const void* act, size_t act_bytes, float* sink,
                                 size_t* delivered_bytes, hipStream_t st) {
  int ng, bt, ks;
  if (d.dtype)
    forward_launch_shape<__bf16>(d, ng, bt, ks);
  else
    forward_launch_shape<float>(d, ng, bt, ks);
  const size_t op = d.op_bytes();
  const dim3 grid((d.HP / 4 + ng - 1) / ng, (d.BP / 16 + bt - 1) / bt);
  // 16-byte vectors per panel, rounded down to whole 1 KiB blocks
  const size_t w_panel = (size_t)ng * 16 * d.KP * op / 1024 * 64;
  const size_t a_panel = ((size_t)bt * 16 * ((size_t)d.KX * 4 + (size_t)d.KH * op)) / 1024 * 64;
  if (w_panel == 0 || a_panel == 0 || a_panel * 16 * grid.y > act_bytes) return hipErrorInvalidValue;
  if ((size_t)grid.x * w_panel * 16 > (size_t)d.G4 * d.KP * op) return hipErrorInvalidValue;
  if (delivered_bytes) *delivered_bytes = (size_t)grid.x * grid.y * (w_panel + a_panel) * 16;
  stream_panels_kernel<<<grid, dim3(64 * ks), 0, st>>>(reinterpret_cast<const uint4*>(Wp), w_panel,
                                                      reinterpret_cast<const uint4*>(act), a_panel, sink);
  return hipGetLastError();
}

template <class T, int NT, int BT, int KS, int U>
static hipError_t launch_backward_cfg(const Dims& d, const BwdParams& p, hipStream_t st) {
  dim3 grid((d.HP / 16 + NT - 1) / NT, (d.BP / 16 + BT - 1) / BT), block(64 * KS);
  backward_kernel<T, NT, BT, KS, U><<<grid, block, 0, st>>>(p);
  return hipGetLastError();
}

template <class T>
static hipError_t launch_backward_t(const Dims& d, const BwdParams& p, hipStream_t st) {
  switch (backward_config<T>(d)) {
    case BWD_SMALLK: return launch_backward_cfg<T, 1, 1, 4, 4>(d, p, st);
    case BWD_22: return launch_backward_cfg<T, 2, 2, 8, 4>(d, p, st);
    case BWD_12: return launch_backward_cfg<T, 1, 2, 8, 6>(d, p, st);
    default: return launch_backward_cfg<T, 1, 1, PAIR_BKS, PAIR_BU>(d, p, st);
  }
}

static BwdParams make_bwd_params(const Dims& d, const BackwardArgs& a) {
  const size_t plane = (size_t)d.B * d.H;
  BwdParams p{};
  p.WTh = a.WTh;
  p.dG_next = a.dG_next;
  p.h = a.state;
  p.c = a.state + d.hplane;
  p.g_i = a.state + d.unit;
  p.g_f = a.state + d.unit + plane;
  p.g_g = a.state + 2 * d.unit;
  p.g_o = a.state + 2 * d.unit + plane;
  p.h_prev = a.prev;
  p.cell = d.cell;
  p.c_prev = a.prev + d.hplane;
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
  p.KH = d.KH;
  p.G4 = d.G4;
  p.NX = d.NX;
  p.KC = d.KC;
  p.BP = d.BP;
  return p;
}

hipError_t launch_backward(const Dims& d, const BackwardArgs& a, hipStream_t st) {
  BwdParams p = make_bwd_params(d, a);
  return d.dtype ? launch_backward_t<__bf16>(d, p, st) : launch_backward_t<float>(d, p, st);
}

// Shape classes for which a fused launch is instantiated: 1 = large K (forward 4 x 1, backward
// 1 x 1, 8 waves each); 2 = small-K forward (4 waves) with the 1 x 2 backward (8 waves).  0 = none.
template <class T>
static int pair_class(const Dims& d) {
  const FwdConfig fc = forward_config<T>(d);
  const BwdConfig bc = backward_config<T>(d);
  if (fc == FWD_B1 && bc == BWD_11) return 1;
  if (fc == FWD_SMALLK && bc == BWD_12) return 2;
  return 0;
}

bool can_fuse_pair(const Dims& d) { return (d.dtype ? pair_class<__bf16>(d) : pair_class<float>(d)) != 0; }

template <class T, int CELL>
static void launch_pair_t(const Dims& d, const FwdParams& f, const BwdParams& b, hipStream_t st) {
  const int nfx = (d.HP / 4 + PAIR_NG - 1) / PAIR_NG, nfy = d.BP / 16;   // both classes: forward 4 x 1
  if (pair_class<T>(d) == 1) {
    const int nbx = d.HP / 16, nby = d.BP / 16;
    pair_kernel<T, CELL, PAIR_NG, PAIR_FKS, PAIR_FU, 1, 1, PAIR_BKS, PAIR_BU>
        <<<dim3(nfx * nfy + nbx * nby), dim3(64 * PAIR_BKS), 0, st>>>(f, b, nfx, nfx * nfy, nbx);
  } else {
    const int nbx = d.HP / 16, nby = (d.BP / 16 + 1) / 2;
    pair_kernel<T, CELL, 4, 4, 1, 1, 2, 8, 2><<<dim3(nfx * nfy + nbx * nby), dim3(512), 0, st>>>(f, b, nfx, nfx * nfy, nbx);
  }
}

hipError_t launch_backward_forward_pair(const Dims& d, const BackwardArgs& a, const void* Wp, const float* bp,
                                        const float* x_s, const float* src_unit, float* dst_unit, float* gates_units,
                                        hipStream_t st) {
  BwdParams b = make_bwd_params(d, a);
  FwdParams f = make_fwd_params(d, Wp, bp, x_s, src_unit, dst_unit, gates_units);
  if (d.dtype)
    d.cell ? launch_pair_t<__bf16, 1>(d, f, b, st) : launch_pair_t<__bf16, 0>(d, f, b, st);
  else
    d.cell ? launch_pair_t<float, 1>(d, f, b, st) : launch_pair_t<float, 0>(d, f, b, st);
  return hipGetLastError();
}

// ---- forward chain with resident weights -----------------------------------------------------
// Consecutive forward operations (Algorithm 2's forward loop; also the single-step pushes that
// follow each other when memory is plentiful) depend on each other only through h, so a chain of
// them can run inside ONE launch if the gate weights stay on the chip and only h travels.  The
// chip is split along the batch: XCD g (one of 8, each with its own L2) takes the sequences
// [g*nb, (g+1)*nb) and never needs anything from another XCD, so no step synchronises across
// XCDs.  Inside an XCD the 32 workgroups (one per compute unit) split the hidden units: workgroup
// `rank` owns units [rank*H/32, (rank+1)*H/32), keeps the 4*H/32 packed weight rows of those units
// in registers (and a part in LDS) for the whole launch, and per step
//   1. waits until all 32 workgroups of its XCD have published their slice of h_{s-1}
//      (a counter in the XCD's L2, bumped with an atomic add and polled with agent-scope loads),
//   2. fetches the bf16 h_{s-1} of its sequences from the exchange ring with loads that bypass the
//      compute unit's vector cache (the ring is written through to the L2 the 32 share),
//   3. runs its slice of the gate GEMM and the pointwise step, keeps c in registers, publishes
//      its slice of h_s, and stores the full state only where the schedule wants one.
// Which XCD a workgroup runs on is read from the hardware (register XCC_ID), not inferred from
// its id: workgroups are dealt round-robin to the XCDs, but where the deal starts depends on the
// launches before.  A workgroup takes the next free rank of its XCD from a counter; the launch
// relies on every XCD receiving exactly 32 of the 256 workgroups, checks it (a rank counter that
// runs past 32 raises the status word; an XCD that gets fewer never completes its first wait,
// which is bounded by a wall-clock limit like every other) and gives up rather than compute on
// an assumption that does not hold.
// Sums are formed exactly as forward_body forms them (KS partial sums over the macro steps
// w, w+KS, ..., added in the order 0..KS-1), so a step gives the same bits either way.
constexpr int RES_MAX_STEPS = 192;  // steps of one launch: their destinations travel as kernel arguments (3 KiB of the 4 KiB there are)
constexpr int RES_RING = 4;         // h slices in flight (two would do: a step ahead at most)
constexpr int RES_WGS = 256, RES_GROUPS = 8, RES_MEMBERS = RES_WGS / RES_GROUPS;
constexpr long long RES_WAIT_TICKS = 50000000;   // 0.5 s of the 100 MHz wall clock
// The bound every wait of a resident launch runs under, in ticks of that clock.  A host-side
// setting (resident_wait_ticks) so that a test can make the waits give up at once -- every
// workgroup then leaves through the same path as after a real time-out -- without anything hanging.
static long long g_wait_ticks = RES_WAIT_TICKS;
void set_resident_wait_ticks(long long ticks) { g_wait_ticks = ticks < 0 ? RES_WAIT_TICKS : ticks; }

struct ResStep {
  float* out;     // unit that receives (h, c) of this step, or NULL
  float* gates;   // two units that receive (i, f), (g, o), or NULL
};
struct ResParams {
  const void* Wp;
  const float* bp;
  const float* x0;     // x of the first step of this launch
  const float* src;    // unit holding the input state of the first step
  void* ring;          // RES_RING x [BP][KH] bf16, fragment-tiled like the 16-bit h plane
  unsigned* sync;      // words: arrival counter of XCD g at [g*64], rank counter at [512 + g*64], status at [1024]
  unsigned base;       // value of every arrival counter when the launch starts
  unsigned launch;     // chain launches of this run before this one (every rank counter stands at 32 * launch)
  long long wait_ticks;   // bound of every wait, in ticks of the 100 MHz wall clock
  int count;
  int B, I, H, KX, KH, BP, nb;
  size_t unit;         // floats per unit
  ResStep step[RES_MAX_STEPS];
};

__device__ inline unsigned xcc_id() {
  unsigned v;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID)" : "=s"(v));
  return v & 0xf;
}

// One operand fragment (16 bytes per lane) fetched with agent scope: the load skips this compute
// unit's vector cache and is served by the XCD's L2, where the other compute units of the XCD have
// just written it.  A buffer load with the scope bit, not an atomic load: the compiler may keep as
// many of them in flight as it has registers for (atomic loads it issues two at a time).
// `base` is wave-uniform; byte_off < 2^31.
__device__ inline bf16x8 load_frag_l2(const void* base, unsigned byte_off) {
  typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
  const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(const_cast<void*>(base), 0, 0x7fffffff, 0x00020000);
  union { u32x4 u; bf16x8 f; } cv;
  cv.u = __builtin_amdgcn_raw_buffer_load_b128(rsrc, (int)byte_off, 0, 16 /* sc1: agent scope */);
  return cv.f;
}

template <int NRT, int NSW, int NSL, int KS, int NBT, int NSXW, int CELL>
__global__ __launch_bounds__(64 * KS) void forward_chain_kernel(ResParams p) {
  using T = __bf16;
  using M = Mma<T>;
  constexpr int VEC = 8, KSTEP = 32, FRAG = 64 * VEC;
  constexpr int NT = NRT * NBT, NSR = NSW - NSL;
  constexpr int UW = NRT * 4, ITEMS = NBT * 16 * UW, NTHR = 64 * KS, IPT = (ITEMS + NTHR - 1) / NTHR;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* red = reinterpret_cast<float*>(smem);                               // [KS][NT][4][64]
  T* wl = reinterpret_cast<T*>(smem + (size_t)KS * NT * 4 * 64 * sizeof(float));   // [KS][NRT][NSL] fragments
  __shared__ int s_go, s_g, s_rank;
  // the wave index as a scalar: conditions on it become scalar branches (an MFMA under a lane mask
  // that is empty would still execute)
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), lane = threadIdx.x & 63;
  const int lrow = lane & 15, lq = lane >> 4;
  if (threadIdx.x == 0) {
    const unsigned xcc = xcc_id();
    int ok = xcc < (unsigned)RES_GROUPS;
    unsigned ticket = 0;
    if (ok) {
      ticket = __hip_atomic_fetch_add(p.sync + 512 + xcc * 64, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      ok = ticket / RES_MEMBERS == p.launch;   // more than 32 workgroups on this XCD: ranks would collide
    }
    if (!ok) __hip_atomic_store(p.sync + 1024, 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_go = ok;
    s_g = ok ? (int)xcc : 0;
    s_rank = (int)(ticket % RES_MEMBERS);
  }
  __syncthreads();
  if (!s_go) return;
  const int g = s_g, rank = s_rank;
  constexpr int nsteps = KS * NSW;
  const int nsx = p.KX / KSTEP, nsh = p.KH / KSTEP;
  const size_t hhalf = (size_t)p.BP * p.KH;
  const int b_lo = g * p.nb, b_hi = min(p.B, b_lo + p.nb);
  const int nbt_all = p.BP / 16;
  const int ct0 = min(b_lo / 16, nbt_all - 1);
  unsigned* ctr = p.sync + g * 64;
  unsigned* status = p.sync + 1024;

  // This workgroup's packed weight rows: row tiles rank*NRT .. +NRT, this wave's macro steps
  // wave, wave + KS, ...; the last NSL of them are parked in LDS (read back by this wave only).
  typename M::Frag wr[NRT][NSR > 0 ? NSR : 1];
  {
    const T* wbase = reinterpret_cast<const T*>(p.Wp) + ((size_t)rank * NRT * nsteps * 64 + lane) * VEC;
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
      for (int i = 0; i < NSW; ++i) {
        const typename M::Frag f = M::load(wbase + ((size_t)rt * nsteps + wave + KS * i) * FRAG);
        if (i < NSR)
          wr[rt][i] = f;
        else
          *reinterpret_cast<typename M::Frag*>(&wl[((size_t)(wave * NRT + rt) * NSL + (i - NSR)) * FRAG + lane * VEC]) = f;
      }
  }

  // Pointwise items of this thread: item = (output tile, lane of the MFMA layout), i.e. the
  // (sequence, unit) whose four gate sums that lane holds, so that the partial sums are read back
  // from LDS at consecutive addresses by consecutive threads.  c stays in registers.
  bool mine[IPT];
  int ib[IPT], iu[IPT], icell[IPT];
  float4 bias[IPT];
  float c_state[IPT];
#pragma unroll
  for (int q = 0; q < IPT; ++q) {
    const int item = (int)threadIdx.x + q * NTHR;
    const int tile = item >> 6, il = item & 63;          // tile = rt * NBT + bt
    const int rt = tile / NBT, bt = tile % NBT;
    const int b = (ct0 + bt) * 16 + (il & 15), u = rank * UW + rt * 4 + (il >> 4);
    mine[q] = item < ITEMS && b >= b_lo && b < b_hi;
    ib[q] = b;
    iu[q] = u;
    icell[q] = tile * 4 * 64 + il;   // where the four gate sums of this item sit inside one wave's block of `red`
    bias[q] = float4{0.f, 0.f, 0.f, 0.f};
    c_state[q] = 0.0f;
    if (mine[q]) {
      bias[q] = *reinterpret_cast<const float4*>(p.bp + 4 * u);
      // the state the pointwise step blends with, kept in this register from step to step:
      // c_{s-1} (LSTM) or h_{s-1} in full precision (GRU)
      c_state[q] = CELL ? HPlane<T>::load(p.src, b, u, nsh, p.H, hhalf) : p.src[hhalf + (size_t)b * p.H + u];
    }
  }
  const bool x_vec = (p.I & 3) == 0;

  // Raw x values of this wave's x macro steps for the step about to run (NSXW = how many of the
  // wave's first steps can fall into the x segment at all: KX / 32 / KS rounded up).
  RawAct<VEC> xraw[NSXW][NBT];
  auto fetch_x = [&](int j) {
    const float* x_j = p.x0 + (size_t)j * p.B * p.I;
#pragma unroll
    for (int i = 0; i < NSXW; ++i) {
      const int s = wave + KS * i;
      if (s < nsx) {
#pragma unroll
        for (int bt = 0; bt < NBT; ++bt) {
          const int b_ld = min(min(ct0 + bt, nbt_all - 1) * 16 + lrow, p.B - 1);
          xraw[i][bt] = load_raw<VEC>(x_j + (size_t)b_ld * p.I, s * KSTEP + VEC * lq, p.I, x_vec);
        }
      }
    }
  };
  fetch_x(0);

  for (int j = 0; j < p.count; ++j) {
    // x fragments: the raw fp32 values were requested a step ahead (see below) and are converted
    // now; they do not depend on the other workgroups
    typename M::Frag bf[NSW][NBT];
#pragma unroll
    for (int i = 0; i < NSXW; ++i)
      if (wave + KS * i < nsx) {
#pragma unroll
        for (int bt = 0; bt < NBT; ++bt) bf[i][bt] = M::from_f32(xraw[i][bt].v);
      }
    f32x4 acc[NRT][NBT];
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
      for (int bt = 0; bt < NBT; ++bt) acc[rt][bt] = f32x4{0.f, 0.f, 0.f, 0.f};
    auto weight = [&](int rt, int i) -> typename M::Frag {
      return (i < NSR) ? wr[rt][i < NSR ? i : 0]
                       : M::load(&wl[((size_t)(wave * NRT + rt) * NSL + (i - NSR)) * FRAG + lane * VEC]);
    };
    // the x part of the sum needs nothing from the other workgroups (a wave's x macro steps precede
    // its h macro steps, so the order of the additions is that of forward_body)
#pragma unroll
    for (int i = 0; i < NSXW; ++i)
      if (wave + KS * i < nsx) {
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) {
          const typename M::Frag a = weight(rt, i);
#pragma unroll
          for (int bt = 0; bt < NBT; ++bt) acc[rt][bt] = M::mma(a, bf[i][bt], acc[rt][bt]);
        }
      }
    if (j > 0) {
      // all 32 workgroups of this XCD have published h of the previous step?
      if (threadIdx.x == 0) {
        const unsigned target = p.base + (unsigned)j * RES_MEMBERS;
        int ok = 1, polls = 0;
        long long t0 = 0;
        // agent-scope loads see the counter in the L2 (32 pollers do not queue behind each other as
        // read-modify-writes would: 1.95 -> 1.59 us per exchange round in isolation)
        while ((int)(__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
          if (p.wait_ticks == 0 || (++polls & 15) == 0) {   // a bound of 0: one look only
            const long long now = wall_clock64();
            if (t0 == 0) t0 = now;
            if (now - t0 >= p.wait_ticks ||
                __hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
              __hip_atomic_store(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              ok = 0;
              break;
            }
          }
        }
        s_go = ok;
      }
      __syncthreads();
      if (!s_go) return;
    }
    // h fragments: the stored input state for the first step, then the exchange ring
    {
      const T* hsrc = (j == 0) ? reinterpret_cast<const T*>(p.src)
                               : reinterpret_cast<const T*>(p.ring) + (size_t)((j - 1) % RES_RING) * hhalf;
#pragma unroll
      for (int i = 0; i < NSW; ++i) {
        const int s = wave + KS * i;
        if (s >= nsx) {
#pragma unroll
          for (int bt = 0; bt < NBT; ++bt) {
            const size_t fo = (((size_t)min(ct0 + bt, nbt_all - 1) * nsh + (s - nsx)) * 64 + lane) * VEC;
            if (j == 0)
              bf[i][bt] = M::load(hsrc + fo);
            else
              bf[i][bt] = load_frag_l2(hsrc, (unsigned)(fo * sizeof(T)));
          }
        }
      }
    }
    __builtin_amdgcn_sched_barrier(0);   // every fetch is issued before the first MFMA
#pragma unroll
    for (int i = 0; i < NSW; ++i)
      if (!(i < NSXW && wave + KS * i < nsx)) {
#pragma unroll
        for (int rt = 0; rt < NRT; ++rt) {
          const typename M::Frag a = weight(rt, i);
#pragma unroll
          for (int bt = 0; bt < NBT; ++bt) acc[rt][bt] = M::mma(a, bf[i][bt], acc[rt][bt]);
        }
      }
    if (j + 1 < p.count) fetch_x(j + 1);   // in flight while this step finishes and the next wait runs
#pragma unroll
    for (int rt = 0; rt < NRT; ++rt)
#pragma unroll
      for (int bt = 0; bt < NBT; ++bt)
#pragma unroll
        for (int r = 0; r < 4; ++r) red[((wave * NT + rt * NBT + bt) * 4 + r) * 64 + lane] = acc[rt][bt][r];
    __syncthreads();
    const ResStep dst = p.step[j];
    T* ring_out = reinterpret_cast<T*>(p.ring) + (size_t)(j % RES_RING) * hhalf;
    const bool publish = j + 1 < p.count;
    float keep_h[IPT], keep_second[IPT], keep_gate[IPT][4];
#pragma unroll
    for (int q = 0; q < IPT; ++q) {
      if (!mine[q]) continue;
      float G[4] = {0.f, 0.f, 0.f, 0.f};
      for (int w = 0; w < KS; ++w)   // fixed order, as in forward_body
#pragma unroll
        for (int r = 0; r < 4; ++r) G[r] += red[w * NT * 4 * 64 + icell[q] + r * 64];
      const float h = cell_forward<CELL>(G, bias[q], c_state[q], keep_second[q], keep_gate[q]);
      keep_h[q] = h;
      c_state[q] = CELL ? h : keep_second[q];
      const int b = ib[q], u = iu[q];
      if (publish) {
        // Units u and u + 1 of one sequence sit 16 lanes apart in this layout and next to each other
        // in the ring: the lane of the even unit stores both as one dword (the rows of a tile belong
        // to one XCD or, split in halves, to two -- a lane and its partner are always on the same side).
        const unsigned hi16 = (__float_as_uint(h) + 0x8000u) >> 16;
        const unsigned other = __shfl_xor(hi16, 16);
        if (((threadIdx.x >> 4) & 1) == 0)
          reinterpret_cast<unsigned*>(ring_out)[ft_offset<T>(b, u, nsh) >> 1] = hi16 | (other << 16);
      }
    }
    if (publish) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's slice of h has reached the L2
      __syncthreads();
      if (threadIdx.x == 0) __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // What only later launches read goes out after the arrival: the other workgroups do not wait
    // for these stores to be acknowledged.
    if (dst.out || dst.gates) {
#pragma unroll
      for (int q = 0; q < IPT; ++q) {
        if (!mine[q]) continue;
        const int b = ib[q], u = iu[q];
        if (dst.out) {
          HPlane<T>::store(dst.out, b, u, keep_h[q], nsh, p.H, hhalf);
          dst.out[hhalf + (size_t)b * p.H + u] = keep_second[q];
        }
        if (dst.gates) {
          const size_t e = (size_t)b * p.H + u, plane = (size_t)p.B * p.H;
          dst.gates[e] = keep_gate[q][0];
          dst.gates[plane + e] = keep_gate[q][1];
          dst.gates[p.unit + e] = keep_gate[q][2];
          if (CELL == 0) dst.gates[p.unit + plane + e] = keep_gate[q][3];
        }
      }
    }
  }
}

// Shape classes with an instantiation: {NRT = H/128, NSW = macro steps per wave, NSL, KS, NBT}.
struct ResConfig {
  int nrt, nsw, nsl, ks, nbt, nsxw;
};
static const ResConfig RES_CONFIGS[] = {
    {8, 5, 1, 8, 1, 1},   // H = 1024, I <= 256
    {4, 5, 0, 4, 1, 1}, {4, 5, 0, 4, 2, 1},   // H = 512, I <= 128
    {2, 4, 0, 4, 1, 2}, {2, 4, 0, 4, 2, 2},   // H = 256, 128 < I <= 256
    {1, 2, 0, 4, 1, 1}, {1, 2, 0, 4, 2, 1},   // H = 128, I <= 128
};

// The batch is dealt to the XCDs in groups of nb consecutive sequences.  An even share,
// nb = ceil(B / 8), keeps every XCD busy but may make a group straddle more 16-sequence MFMA tiles
// than a kernel is instantiated for; the share rounded up to whole tiles never straddles (some XCDs
// then get no sequences and only keep the meeting going).  group_tiles: batch tiles the widest group
// touches; the configuration look-ups try the even share first.
static int group_tiles(const Dims& d, int nb) {
  int nbt = 1;
  for (int g = 0; g < RES_GROUPS; ++g) {
    const int lo = g * nb, hi = (lo + nb < d.B ? lo + nb : d.B);
    if (lo >= d.B) break;
    const int span = (hi - 1) / 16 - lo / 16 + 1;
    nbt = span > nbt ? span : nbt;
  }
  return nbt;
}
static int group_share(const Dims& d, int candidate) {
  const int even = (d.B + RES_GROUPS - 1) / RES_GROUPS;
  return candidate == 0 ? even : round_up(even, 16);
}

// Index into RES_CONFIGS for this shape, or -1 when the chain kernel does not apply; *nb_out = the
// sequences per XCD to launch it with.
static int resident_config(const Dims& d, int* nb_out = nullptr) {
  if (!d.dtype || d.H % 128 != 0 || d.KH != d.H) return -1;   // either cell: the GRU's rows r, z, n_x, n_h fill the same four packed rows
  const int nsteps = d.KP / 32;
  const FwdConfig fc = forward_config<__bf16>(d);
  const int ks = (fc == FWD_TINY || fc == FWD_SMALLK) ? 4 : 8;   // the K split of the per-step kernels
  if (nsteps % ks != 0) return -1;
  for (int cand = 0; cand < 2; ++cand) {
    const int nb = group_share(d, cand), nbt = group_tiles(d, nb);
    for (size_t i = 0; i < sizeof RES_CONFIGS / sizeof RES_CONFIGS[0]; ++i) {
      const ResConfig& c = RES_CONFIGS[i];
      if (c.nrt == d.H / 128 && c.ks == ks && c.nsw == nsteps / ks && c.nbt == nbt && c.nsxw == (d.KX / 32 + ks - 1) / ks) {
        if (nb_out) *nb_out = nb;
        return (int)i;
      }
    }
  }
  return -1;
}

bool can_run_forward_chain(const Dims& d) { return resident_config(d) >= 0; }
int forward_chain_max_steps() { return RES_MAX_STEPS; }
size_t forward_chain_ring_bytes(const Dims& d) { return (size_t)RES_RING * d.BP * d.KH * sizeof(__bf16); }
size_t forward_chain_sync_bytes() { return (1024 + 64) * sizeof(unsigned); }
size_t forward_chain_status_offset() { return 1024 * sizeof(unsigned); }
unsigned forward_chain_arrivals(int steps) { return steps > 1 ? (unsigned)(steps - 1) * RES_MEMBERS : 0u; }

template <int NRT, int NSW, int NSL, int KS, int NBT, int NSXW, int CELL>
static hipError_t launch_chain_cell(const ResParams& p, hipStream_t st) {
  const size_t lds = (size_t)KS * NRT * NBT * 4 * 64 * sizeof(float) + (size_t)KS * NRT * NSL * 64 * 8 * sizeof(__bf16);
  static bool configured = false;   // per instantiation; the attribute only has to be set once
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(forward_chain_kernel<NRT, NSW, NSL, KS, NBT, NSXW, CELL>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  forward_chain_kernel<NRT, NSW, NSL, KS, NBT, NSXW, CELL><<<dim3(RES_WGS), dim3(64 * KS), lds, st>>>(p);
  return hipGetLastError();
}
template <int NRT, int NSW, int NSL, int KS, int NBT, int NSXW>
static hipError_t launch_chain_cfg(const ResParams& p, int cell, hipStream_t st) {
  return cell ? launch_chain_cell<NRT, NSW, NSL, KS, NBT, NSXW, 1>(p, st) : launch_chain_cell<NRT, NSW, NSL, KS, NBT, NSXW, 0>(p, st);
}

hipError_t launch_forward_chain(const Dims& d, const void* Wp, const float* bp, const float* x_first, const float* src_unit,
                                const ChainStep* steps, int count, void* ring, unsigned* sync, unsigned base,
                                unsigned launch, hipStream_t st) {
  int nb = 0;
  const int cfg = resident_config(d, &nb);
  if (cfg < 0 || count < 1 || count > RES_MAX_STEPS) return hipErrorInvalidValue;
  ResParams p{};
  p.Wp = Wp;
  p.bp = bp;
  p.x0 = x_first;
  p.src = src_unit;
  p.ring = ring;
  p.sync = sync;
  p.base = base;
  p.launch = launch;
  p.wait_ticks = g_wait_ticks;
  p.count = count;
  p.B = d.B;
  p.I = d.I;
  p.H = d.H;
  p.KX = d.KX;
  p.KH = d.KH;
  p.BP = d.BP;
  p.nb = nb;
  p.unit = d.unit;
  for (int j = 0; j < count; ++j) p.step[j] = ResStep{steps[j].out, steps[j].gates};
  switch (cfg) {
    case 0: return launch_chain_cfg<8, 5, 1, 8, 1, 1>(p, d.cell, st);
    case 1: return launch_chain_cfg<4, 5, 0, 4, 1, 1>(p, d.cell, st);
    case 2: return launch_chain_cfg<4, 5, 0, 4, 2, 1>(p, d.cell, st);
    case 3: return launch_chain_cfg<2, 4, 0, 4, 1, 2>(p, d.cell, st);
    case 4: return launch_chain_cfg<2, 4, 0, 4, 2, 2>(p, d.cell, st);
    case 5: return launch_chain_cfg<1, 2, 0, 4, 1, 1>(p, d.cell, st);
    default: return launch_chain_cfg<1, 2, 0, 4, 2, 1>(p, d.cell, st);
  }
}

// ---- backward sweep with resident weights ------------------------------------------------------
// Where a sub-sequence fits into memory the schedule alternates "forward operation of step s from
// the memorised h_{s-1}, keeping the internal state" and "backward operation of step s", s going
// down.  On shapes whose gate weights AND their transpose fit on the chip such a run of pairs goes
// out as one launch per chunk of steps, organised like the forward chain (batch split over the
// XCDs, hidden units over the 32 compute units of an XCD, weights in registers):
//   * the forward operation of a step needs nothing from other compute units (its input state was
//     memorised by an earlier launch), and its internal state never leaves the registers of the
//     thread that owns the (sequence, unit);
//   * the backward operation needs dG of the step after, all 4H columns of it, for the XCD's
//     sequences: the compute units publish their columns in the chunk's dG staging buffer (which
//     is already laid out as that GEMM's operand) and meet at the XCD's arrival counter;
//   * while the counter fills, every compute unit already runs the forward operation of the next
//     lower step, so the wait is mostly hidden.
// K splits and summation orders are those of forward_body and backward_body for the shape, the
// pointwise steps are the shared functions: bit-identical to the launch-per-step path.
constexpr int SWEEP_MAX_STEPS = 32;
struct SweepParams {
  const void* Wp;
  const void* WTh;
  const float* bp;
  const float* x;        // x of step 1 (step s reads x + (s-1)*B*I)
  const float* dy;       // upstream gradients, first plane = step dy_first; NULL with dy_is_h
  int dy_first, dy_is_h;
  float* dc;             // running cell-state gradient plane
  float* y_out;          // outputs, plane of step 1 first, or NULL
  const void* dG_next;   // dG block of step s_hi + 1, or NULL when s_hi is the last step of the sequence
  void* dG_chunk[2];     // the two chunk buffers: step s lives in buffer ((s-1) / CH) & 1, its block at slot (s-1) % CH
  void* dGT[2];
  void* aT[2];
  unsigned* sync;
  unsigned base, launch;
  long long wait_ticks;  // bound of every wait, in ticks of the 100 MHz wall clock
  int s_hi, count;       // steps s_hi, s_hi - 1, ..., s_hi - count + 1 (in at most two consecutive chunks)
  int B, I, H, KX, KH, BP, nb, G4, NX, KC, CH;
  size_t unit;
  const float* src[SWEEP_MAX_STEPS];   // src[j]: unit holding the state before step s_hi - j
  const float* state[SWEEP_MAX_STEPS]; // FWD = false: unit holding the stored internal state of step s_hi - j
};

// FWD = false: the internal states are not recomputed but read from where an earlier launch
// stored them (internal-state slots): a run of backward operations only, W_hh^T alone resident.
template <bool FWD, int NRT, int NSWF, int KSF, int NSWB, int KSB, int NBT, int NSXW, int CELL = 0>
__global__ __launch_bounds__(512) void sweep_kernel(SweepParams p) {
  static_assert(!(FWD && CELL), "the launches that recompute internal states are built for the LSTM only");
  using T = __bf16;
  using M = Mma<T>;
  constexpr int VEC = 8, KSTEP = 32;
  constexpr int FT = 8 / KSF;                       // groups of waves that split the forward row tiles
  constexpr int NRTW = (NRT + FT - 1) / FT;         // forward row tiles per wave
  constexpr int UW = NRT * 4;                       // hidden units per workgroup
  constexpr int NTB = (UW + 15) / 16;               // 16-unit tiles of the dh GEMM that cover them
  constexpr int NTF = NRT * NBT, NTBT = NTB * NBT;
  constexpr int ITEMS = NRT * NBT * 64, IPT = (ITEMS + 511) / 512;
  constexpr int nstepsF = KSF * NSWF, nstepsB = KSB * NSWB;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  float* redF = reinterpret_cast<float*>(smem);                       // [KSF][NTF][4][64]
  float* redB = redF + (size_t)KSF * NTF * 4 * 64;                    // [KSB][NTBT][4][64]
  __shared__ int s_go, s_g, s_rank;
  // the wave index as a scalar: conditions on it become scalar branches (an MFMA under a lane mask
  // that is empty would still execute)
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), lane = threadIdx.x & 63;
  const int lrow = lane & 15, lq = lane >> 4;
  if (threadIdx.x == 0) {
    const unsigned xcc = xcc_id();
    int ok = xcc < (unsigned)RES_GROUPS;
    unsigned ticket = 0;
    if (ok) {
      ticket = __hip_atomic_fetch_add(p.sync + 512 + xcc * 64, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      ok = ticket / RES_MEMBERS == p.launch;
    }
    if (!ok) __hip_atomic_store(p.sync + 1024, 2u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    s_go = ok;
    s_g = ok ? (int)xcc : 0;
    s_rank = (int)(ticket % RES_MEMBERS);
  }
  __syncthreads();
  if (!s_go) return;
  const int g = s_g, rank = s_rank;
  const int nsx = p.KX / KSTEP, nsh = p.KH / KSTEP;
  const size_t hhalf = (size_t)p.BP * p.KH, plane = (size_t)p.B * p.H;
  const int b_lo = g * p.nb, b_hi = min(p.B, b_lo + p.nb);
  const int nbt_all = p.BP / 16;
  const int ct0 = min(b_lo / 16, nbt_all - 1);
  unsigned* ctr = p.sync + g * 64;
  unsigned* status = p.sync + 1024;
  const int fk = wave % KSF, fg = wave / KSF;       // forward: K part and row-tile group of this wave
  const bool bwd_wave = wave < KSB;
  const int nt0 = (rank * UW) / 16;                 // first 16-unit tile of the dh GEMM

  // resident weights: forward rows of this workgroup's units, and the rows of W_hh^T for the same units
  typename M::Frag wf[FWD ? NRTW : 1][FWD ? NSWF : 1], wb[NTB][NSWB];
  if (FWD) {
#pragma unroll
    for (int i = 0; i < NRTW; ++i) {
      const int rt = min(fg * NRTW + i, NRT - 1);
#pragma unroll
      for (int k = 0; k < NSWF; ++k)
        wf[FWD ? i : 0][FWD ? k : 0] = M::load(reinterpret_cast<const T*>(p.Wp) +
                                               (((size_t)(rank * NRT + rt) * nstepsF + fk + KSF * k) * 64 + lane) * VEC);
    }
  }
#pragma unroll
  for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
    for (int k = 0; k < NSWB; ++k)
      wb[tb][k] = M::load(reinterpret_cast<const T*>(p.WTh) +
                          (((size_t)(nt0 + tb) * nstepsB + min(wave, KSB - 1) + KSB * k) * 64 + lane) * VEC);

  // items: (output tile, lane of the forward MFMA layout) = (sequence, unit)
  bool mine[IPT];
  int ib[IPT], iu[IPT], icellF[IPT], icellB[IPT];
  float4 bias[IPT];
  float dc_run[IPT];
  // internal state of the step whose backward operation comes next, and its input state
  float st_gate[IPT][4], st_c[IPT], st_h[IPT], st_cprev[IPT], st_hprev[IPT];
#pragma unroll
  for (int q = 0; q < IPT; ++q) {
    const int item = (int)threadIdx.x + q * 512;
    const int tile = item >> 6, il = item & 63;
    const int rt = tile / NBT, bt = tile % NBT;
    const int b = (ct0 + bt) * 16 + (il & 15), u = rank * UW + rt * 4 + (il >> 4);
    mine[q] = item < ITEMS && b >= b_lo && b < b_hi;
    ib[q] = b;
    iu[q] = u;
    icellF[q] = tile * 4 * 64 + il;
    // dh of unit u: row u % 16 of tile u / 16 of the dh GEMM, i.e. lane (u%16/4)*16 + b%16, register u%4
    icellB[q] = (((u / 16 - nt0) * NBT + bt) * 4 + (u & 3)) * 64 + ((u & 15) >> 2) * 16 + (il & 15);
    bias[q] = float4{0.f, 0.f, 0.f, 0.f};
    dc_run[q] = 0.0f;
    if (mine[q]) {
      bias[q] = *reinterpret_cast<const float4*>(p.bp + 4 * u);
      dc_run[q] = p.dc[(size_t)b * p.H + u];
    }
  }
  // operands of a forward operation, requested a step ahead: raw x values, h fragments, c_{s-1}, h_{s-1}
  RawAct<VEC> xraw[FWD ? NSXW : 1][NBT];
  typename M::Frag hfr[FWD ? NSWF : 1][NBT];
  float pf_cprev[IPT], pf_hprev[IPT];
  float pf_gate[FWD ? 1 : IPT][4], pf_c[FWD ? 1 : IPT], pf_h[FWD ? 1 : IPT];   // FWD = false: the stored state, a step ahead
  const bool want_h = p.dy_is_h || p.y_out != nullptr;
  auto fetch_fwd = [&](int j) {
    if (!FWD) {
      const float* stp = p.state[j];
      const float* src = p.src[j];
#pragma unroll
      for (int q = 0; q < IPT; ++q) {
        pf_cprev[q] = pf_hprev[q] = 0.0f;
        pf_c[FWD ? 0 : q] = pf_h[FWD ? 0 : q] = 0.0f;
#pragma unroll
        for (int r = 0; r < 4; ++r) pf_gate[FWD ? 0 : q][r] = 0.0f;
        if (mine[q]) {
          const size_t e = (size_t)ib[q] * p.H + iu[q];
          pf_gate[FWD ? 0 : q][0] = stp[p.unit + e];
          pf_gate[FWD ? 0 : q][1] = stp[p.unit + plane + e];
          pf_gate[FWD ? 0 : q][2] = stp[2 * p.unit + e];
          if (CELL == 0) pf_gate[FWD ? 0 : q][3] = stp[2 * p.unit + plane + e];   // the GRU has three gates
          pf_c[FWD ? 0 : q] = stp[hhalf + e];                                     // c_s, or the GRU's n_h
          if (want_h) pf_h[FWD ? 0 : q] = HPlane<T>::load(stp, ib[q], iu[q], nsh, p.H, hhalf);
          // what the pointwise step blends with: c_{s-1}, or the GRU's h_{s-1} in full precision
          pf_cprev[q] = CELL ? HPlane<T>::load(src, ib[q], iu[q], nsh, p.H, hhalf) : src[hhalf + e];
          pf_hprev[q] = (float)HPlane<T>::as_operand(src, ib[q], iu[q], nsh, p.H, hhalf);
        }
      }
      return;
    }
    const int s = p.s_hi - j;
    const float* x_s = p.x + (size_t)(s - 1) * p.B * p.I;
    const float* src = p.src[j];
#pragma unroll
    for (int k = 0; k < NSWF; ++k) {
      const int ms = fk + KSF * k;
#pragma unroll
      for (int bt = 0; bt < NBT; ++bt) {
        const int tile = min(ct0 + bt, nbt_all - 1);
        if (ms < nsx) {
          if (k < NSXW) xraw[(FWD && k < NSXW) ? k : 0][bt] = load_raw_whole<VEC>(x_s + (size_t)min(tile * 16 + lrow, p.B - 1) * p.I,
                                                                                  ms * KSTEP + VEC * lq, p.I);
        } else {
          hfr[FWD ? k : 0][bt] = M::load(reinterpret_cast<const T*>(src) + (((size_t)tile * nsh + (ms - nsx)) * 64 + lane) * VEC);
        }
      }
    }
#pragma unroll
    for (int q = 0; q < IPT; ++q) {
      pf_cprev[q] = pf_hprev[q] = 0.0f;
      if (mine[q]) {
        pf_cprev[q] = src[hhalf + (size_t)ib[q] * p.H + iu[q]];
        pf_hprev[q] = (float)HPlane<T>::as_operand(src, ib[q], iu[q], nsh, p.H, hhalf);
      }
    }
  };
  // The forward operation of step s_hi - j comes in two parts, so that the memory operations
  // between them overlap with neither's waits.  (Loads and stores share one in-order counter: once
  // both kinds are in flight, a wait for any load is a wait for everything, store acknowledgements
  // included.)  Part one runs right after an arrival, when nothing is outstanding: the GEMM slice
  // from the fetched operands, then the request for the operands of the step after.  Part two, after
  // the stores that only later launches read have been issued, reduces the slices and applies the
  // gate functions; it leaves the internal state in st_*.
  auto forward_gemm = [&](int j) {
#pragma unroll
    for (int q = 0; q < IPT; ++q) {
      st_cprev[q] = pf_cprev[q];
      st_hprev[q] = pf_hprev[q];
      if (!FWD) {   // nothing to compute: the fetched state becomes the current one
#pragma unroll
        for (int r = 0; r < 4; ++r) st_gate[q][r] = pf_gate[FWD ? 0 : q][r];
        st_c[q] = pf_c[FWD ? 0 : q];
        st_h[q] = pf_h[FWD ? 0 : q];
      }
    }
    if (FWD) {
      f32x4 acc[NRTW][NBT];
#pragma unroll
      for (int i = 0; i < NRTW; ++i)
#pragma unroll
        for (int bt = 0; bt < NBT; ++bt) acc[i][bt] = f32x4{0.f, 0.f, 0.f, 0.f};
#pragma unroll
      for (int k = 0; k < NSWF; ++k) {
        const int ms = fk + KSF * k;
#pragma unroll
        for (int bt = 0; bt < NBT; ++bt) {
          const typename M::Frag bfr = (k < NSXW && ms < nsx) ? M::from_f32(xraw[(FWD && k < NSXW) ? k : 0][bt].v) : hfr[FWD ? k : 0][bt];
#pragma unroll
          for (int i = 0; i < NRTW; ++i) acc[i][bt] = M::mma(wf[FWD ? i : 0][FWD ? k : 0], bfr, acc[i][bt]);
        }
      }
#pragma unroll
      for (int i = 0; i < NRTW; ++i) {
        const int rt = fg * NRTW + i;
        if (rt < NRT) {
#pragma unroll
          for (int bt = 0; bt < NBT; ++bt)
#pragma unroll
            for (int r = 0; r < 4; ++r) redF[((fk * NTF + rt * NBT + bt) * 4 + r) * 64 + lane] = acc[i][bt][r];
        }
      }
    }
    if (j + 1 < p.count) fetch_fwd(j + 1);
  };
  auto forward_point = [&]() {
    if (!FWD) return;
    __syncthreads();
#pragma unroll
    for (int q = 0; q < IPT; ++q) {
      if (!mine[q]) continue;
      float G[4] = {0.f, 0.f, 0.f, 0.f};
      for (int w = 0; w < KSF; ++w)   // fixed order, as in forward_body
#pragma unroll
        for (int r = 0; r < 4; ++r) G[r] += redF[w * NTF * 4 * 64 + icellF[q] + r * 64];
      float second;
      st_h[q] = cell_forward<0>(G, bias[q], st_cprev[q], second, st_gate[q]);
      st_c[q] = second;
    }
  };

  fetch_fwd(0);
  forward_gemm(0);   // also requests the operands of the step after
  forward_point();

  for (int j = 0; j < p.count; ++j) {
    const int s = p.s_hi - j;                       // the step back-propagated now
    const int slot = (s - 1) % p.CH, buf = ((s - 1) / p.CH) & 1;   // where step s lives in the chunk buffers
    const size_t dG_step = (size_t)p.BP * p.G4;     // elements of one step's dG block
    const T* dG_next = (j == 0) ? reinterpret_cast<const T*>(p.dG_next)   // step s + 1: maybe in the other buffer
                                : reinterpret_cast<const T*>(p.dG_chunk[(s / p.CH) & 1]) + (size_t)(s % p.CH) * dG_step;
    if (j > 0) {
      // all 32 workgroups of this XCD have published their columns of dG of step s + 1?
      if (threadIdx.x == 0) {
        const unsigned target = p.base + (unsigned)j * RES_MEMBERS;
        int ok = 1, polls = 0;
        long long t0 = 0;
        while ((int)(__hip_atomic_load(ctr, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) - target) < 0) {
          if (p.wait_ticks == 0 || (++polls & 15) == 0) {   // a bound of 0: one look only
            const long long now = wall_clock64();
            if (t0 == 0) t0 = now;
            if (now - t0 >= p.wait_ticks ||
                __hip_atomic_load(status, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT) != 0u) {
              __hip_atomic_store(status, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
              ok = 0;
              break;
            }
          }
        }
        s_go = ok;
      }
      __syncthreads();
      if (!s_go) return;
    }
    // dh = dG_{s+1} W_hh for this workgroup's units
    if (dG_next != nullptr) {
      if (bwd_wave) {
        f32x4 acc[NTB][NBT];
#pragma unroll
        for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
          for (int bt = 0; bt < NBT; ++bt) acc[tb][bt] = f32x4{0.f, 0.f, 0.f, 0.f};
        // The dG fragments come in rounds of GK macro steps: all fetches of a round go out before its
        // first MFMA (left to itself the scheduler pairs each fetch with the MFMA that needs it, one
        // L2 round trip after the other).  Two batch tiles beside resident forward weights leave
        // registers for half the fragments at a time only.
        constexpr int GK = (FWD && NBT > 1) ? NSWB / 2 : NSWB;
#pragma unroll
        for (int k0 = 0; k0 < NSWB; k0 += GK) {
          typename M::Frag gfr[GK][NBT];
#pragma unroll
          for (int k = 0; k < GK; ++k)
#pragma unroll
            for (int bt = 0; bt < NBT; ++bt) {
              const size_t fo = (((size_t)min(ct0 + bt, nbt_all - 1) * nstepsB + wave + KSB * (k0 + k)) * 64 + lane) * VEC;
              gfr[k][bt] = load_frag_l2(dG_next, (unsigned)(fo * sizeof(T)));
            }
          __builtin_amdgcn_sched_barrier(0);
#pragma unroll
          for (int k = 0; k < GK; ++k)
#pragma unroll
            for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
              for (int bt = 0; bt < NBT; ++bt) acc[tb][bt] = M::mma(wb[tb][k0 + k], gfr[k][bt], acc[tb][bt]);
          __builtin_amdgcn_sched_barrier(0);
        }
#pragma unroll
        for (int tb = 0; tb < NTB; ++tb)
#pragma unroll
          for (int bt = 0; bt < NBT; ++bt)
#pragma unroll
            for (int r = 0; r < 4; ++r) redB[((wave * NTBT + tb * NBT + bt) * 4 + r) * 64 + lane] = acc[tb][bt][r];
      }
      __syncthreads();
    }
    // pointwise backward of step s on the internal state held in registers
    const bool publish = j + 1 < p.count;
    T* dG_cur = reinterpret_cast<T*>(p.dG_chunk[buf]) + (size_t)slot * dG_step;
    const int ncs = p.KC / KSTEP, col0 = slot * p.B;
    T gq[IPT][4];
    float keep_h[IPT], keep_hprev[IPT];
#pragma unroll
    for (int q = 0; q < IPT; ++q) {
      if (!mine[q]) continue;
      const int b = ib[q], n = iu[q];
      const size_t e = (size_t)b * p.H + n;
      float dh = 0.0f;
      if (dG_next != nullptr)
        for (int w = 0; w < KSB; ++w) dh += redB[w * NTBT * 4 * 64 + icellB[q]];   // fixed order, as in backward_body
      float dyv = 0.0f;
      if (p.dy_is_h)
        dyv = st_h[q];
      else if (p.dy != nullptr && s >= p.dy_first)
        dyv = p.dy[(size_t)(s - p.dy_first) * plane + e];
      dh += dyv;
      float dG[4], dc_out;
      if (CELL == 0)
        lstm_backward_point(dh, dc_run[q], st_gate[q][0], st_gate[q][1], st_gate[q][2], st_gate[q][3], st_c[q], st_cprev[q],
                            dG, dc_out);
      else   // the running plane carries dh_{s+1} * z_{s+1}, as in backward_body
        gru_backward_point(__fadd_rn(dh, dc_run[q]), st_gate[q][0], st_gate[q][1], st_gate[q][2], st_c[q], st_cprev[q], dG, dc_out);
      dc_run[q] = dc_out;
      // the four gates of a unit are consecutive in dG: one 8-byte store (what other compute units
      // fetch next must not be written in pieces smaller than a dword)
      union { T t[4]; unsigned long long v; } pk;
#pragma unroll
      for (int r = 0; r < 4; ++r) pk.t[r] = gq[q][r] = (T)dG[r];
      *reinterpret_cast<unsigned long long*>(dG_cur + ft_offset<T>(b, 4 * n, nstepsB)) = pk.v;
      keep_h[q] = st_h[q];
      keep_hprev[q] = st_hprev[q];
    }
    if (publish) {
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");   // this thread's columns of dG have reached the L2
      __syncthreads();
      if (threadIdx.x == 0) __hip_atomic_fetch_add(ctr, 1u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      forward_gemm(j + 1);
    }
    // What only later launches read -- the transposed copies for the weight gradient, the output --
    // is stored after the arrival: nobody in this launch waits for it.
#pragma unroll
    for (int q = 0; q < IPT; ++q) {
      if (!mine[q]) continue;
      const int b = ib[q], n = iu[q];
      const int col = col0 + b;
      T* dGT = reinterpret_cast<T*>(p.dGT[buf]);
#pragma unroll
      for (int r = 0; r < 4; ++r) dGT[ft_offset<T>(4 * n + r, col, ncs)] = gq[q][r];
      reinterpret_cast<T*>(p.aT[buf])[ft_offset<T>(p.NX + n, col, ncs)] = (T)keep_hprev[q];
      if (p.y_out) p.y_out[(size_t)(s - 1) * plane + (size_t)b * p.H + n] = keep_h[q];
    }
    // the pointwise part of the next lower step's forward operation runs while the others arrive
    if (publish) forward_point();
  }
#pragma unroll
  for (int q = 0; q < IPT; ++q)
    if (mine[q]) p.dc[(size_t)ib[q] * p.H + iu[q]] = dc_run[q];
}

struct SweepConfig {
  int nrt, nswf, ksf, nswb, ksb, nbt, nsxw;
};
static const SweepConfig SWEEP_CONFIGS[] = {
    {4, 5, 4, 8, 8, 1, 1}, {4, 5, 4, 8, 8, 2, 1},   // H = 512, I <= 128
    {2, 4, 4, 4, 8, 1, 2}, {2, 4, 4, 4, 8, 2, 2},   // H = 256, 128 < I <= 256
    {1, 2, 4, 4, 4, 1, 1}, {1, 2, 4, 4, 4, 2, 1},   // H = 128, I <= 128
    {8, 5, 8, 16, 8, 1, 1},                         // H = 1024, any I: backward operations only (W_hh^T fits, both do not)
};
constexpr int SWEEP_BACKWARD_ONLY_FROM = 6;   // configurations from this index on have no forward part

// backward_only: for a launch of backward operations on stored internal states, which never reads x
// or the gate weights -- only the backward part of a configuration has to fit the shape.
static int sweep_config(const Dims& d, int* nb_out = nullptr, bool backward_only = false) {
  if (!d.dtype || d.H % 128 != 0 || d.KH != d.H || d.HP != d.H) return -1;   // either cell; can_run_sweep() narrows
  const int nstepsF = d.KP / 32, nstepsB = d.G4 / 32;
  const FwdConfig fc = forward_config<__bf16>(d);
  const int ksf = (fc == FWD_TINY || fc == FWD_SMALLK) ? 4 : 8;
  const int ksb = backward_config<__bf16>(d) == BWD_SMALLK ? 4 : 8;
  if (nstepsB % ksb != 0) return -1;
  for (int cand = 0; cand < 2; ++cand) {
    const int nb = group_share(d, cand), nbt = group_tiles(d, nb);
    for (size_t i = 0; i < sizeof SWEEP_CONFIGS / sizeof SWEEP_CONFIGS[0]; ++i) {
      const SweepConfig& c = SWEEP_CONFIGS[i];
      if (c.nrt != d.H / 128 || c.ksb != ksb || c.nswb != nstepsB / ksb || c.nbt != nbt) continue;
      // the forward part fixes the width of x as well
      if (backward_only || (int)i >= SWEEP_BACKWARD_ONLY_FROM ||
          (d.I % 8 == 0 && nstepsF % ksf == 0 && c.ksf == ksf && c.nswf == nstepsF / ksf &&
           c.nsxw == (d.KX / 32 + ksf - 1) / ksf)) {
        if (nb_out) *nb_out = nb;
        return (int)i;
      }
    }
  }
  return -1;
}

bool can_run_sweep(const Dims& d) {   // with forward operations: LSTM only
  const int c = sweep_config(d);
  return d.cell == 0 && c >= 0 && c < SWEEP_BACKWARD_ONLY_FROM;
}
bool can_run_backward_sweep(const Dims& d) { return sweep_config(d, nullptr, true) >= 0; }
int sweep_max_steps() { return SWEEP_MAX_STEPS; }

template <bool FWD, int NRT, int NSWF, int KSF, int NSWB, int KSB, int NBT, int NSXW, int CELL = 0>
static hipError_t launch_sweep_cfg(const SweepParams& p, hipStream_t st) {
  constexpr int NTB = (NRT * 4 + 15) / 16;
  const size_t lds = ((size_t)KSF * NRT * NBT + (size_t)KSB * NTB * NBT) * 4 * 64 * sizeof(float);
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(sweep_kernel<FWD, NRT, NSWF, KSF, NSWB, KSB, NBT, NSXW, CELL>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  sweep_kernel<FWD, NRT, NSWF, KSF, NSWB, KSB, NBT, NSXW, CELL><<<dim3(RES_WGS), dim3(512), lds, st>>>(p);
  return hipGetLastError();
}

hipError_t launch_sweep(const Dims& d, const SweepArgs& a, hipStream_t st) {
  int nb = 0;
  const int cfg = sweep_config(d, &nb, a.state != nullptr);
  if (cfg < 0 || a.count < 1 || a.count > SWEEP_MAX_STEPS) return hipErrorInvalidValue;
  if ((a.s_hi - 1) / d.CH - (a.s_hi - a.count) / d.CH > 1) return hipErrorInvalidValue;   // two chunk buffers
  SweepParams p{};
  p.Wp = a.Wp;
  p.WTh = a.WTh;
  p.bp = a.bp;
  p.x = a.x;
  p.dy = a.dy;
  p.dy_first = a.dy_first;
  p.dy_is_h = a.dy_is_h;
  p.dc = a.dc;
  p.y_out = a.y_out;
  p.dG_next = a.dG_next;
  for (int i = 0; i < 2; ++i) {
    p.dG_chunk[i] = a.dG_chunk[i];
    p.dGT[i] = a.dGT[i];
    p.aT[i] = a.aT[i];
  }
  p.sync = a.sync;
  p.base = a.base;
  p.wait_ticks = g_wait_ticks;
  p.launch = a.launch;
  p.s_hi = a.s_hi;
  p.count = a.count;
  p.B = d.B;
  p.I = d.I;
  p.H = d.H;
  p.KX = d.KX;
  p.KH = d.KH;
  p.BP = d.BP;
  p.nb = nb;
  p.G4 = d.G4;
  p.NX = d.NX;
  p.KC = d.KC;
  p.CH = d.CH;
  p.unit = d.unit;
  for (int j = 0; j < a.count; ++j) {
    p.src[j] = a.src[j];
    p.state[j] = a.state ? a.state[j] : nullptr;
  }
  if (a.state) {   // backward operations through stored internal states
    if (d.cell)
      switch (cfg) {
        case 0: return launch_sweep_cfg<false, 4, 5, 4, 8, 8, 1, 1, 1>(p, st);
        case 1: return launch_sweep_cfg<false, 4, 5, 4, 8, 8, 2, 1, 1>(p, st);
        case 2: return launch_sweep_cfg<false, 2, 4, 4, 4, 8, 1, 2, 1>(p, st);
        case 3: return launch_sweep_cfg<false, 2, 4, 4, 4, 8, 2, 2, 1>(p, st);
        case 4: return launch_sweep_cfg<false, 1, 2, 4, 4, 4, 1, 1, 1>(p, st);
        case 5: return launch_sweep_cfg<false, 1, 2, 4, 4, 4, 2, 1, 1>(p, st);
        default: return launch_sweep_cfg<false, 8, 5, 8, 16, 8, 1, 1, 1>(p, st);
      }
    switch (cfg) {
      case 0: return launch_sweep_cfg<false, 4, 5, 4, 8, 8, 1, 1>(p, st);
      case 1: return launch_sweep_cfg<false, 4, 5, 4, 8, 8, 2, 1>(p, st);
      case 2: return launch_sweep_cfg<false, 2, 4, 4, 4, 8, 1, 2>(p, st);
      case 3: return launch_sweep_cfg<false, 2, 4, 4, 4, 8, 2, 2>(p, st);
      case 4: return launch_sweep_cfg<false, 1, 2, 4, 4, 4, 1, 1>(p, st);
      case 5: return launch_sweep_cfg<false, 1, 2, 4, 4, 4, 2, 1>(p, st);
      default: return launch_sweep_cfg<false, 8, 5, 8, 16, 8, 1, 1>(p, st);
    }
  }
  if (d.cell || cfg >= SWEEP_BACKWARD_ONLY_FROM) return hipErrorInvalidValue;
  switch (cfg) {
    case 0: return launch_sweep_cfg<true, 4, 5, 4, 8, 8, 1, 1>(p, st);
    case 1: return launch_sweep_cfg<true, 4, 5, 4, 8, 8, 2, 1>(p, st);
    case 2: return launch_sweep_cfg<true, 2, 4, 4, 4, 8, 1, 2>(p, st);
    case 3: return launch_sweep_cfg<true, 2, 4, 4, 4, 8, 2, 2>(p, st);
    case 4: return launch_sweep_cfg<true, 1, 2, 4, 4, 4, 1, 1>(p, st);
    case 5: return launch_sweep_cfg<true, 1, 2, 4, 4, 4, 2, 1>(p, st);
    default: return hipErrorInvalidValue;
  }
}

// ---- data-gradient GEMM: out[row][n] = sum_k dG[row][k] * WT[n][k] ---------------------------

// One workgroup = NT column tiles (16 outputs n each) x RT row tiles (16 (step, sequence) rows each);
// its KS waves split K = 4*HP, every wave covering all NT x RT tiles.  Partial sums meet in LDS;
// the NT*RT*4 output quarter-tiles are dealt round-robin to the waves for the store.
template <class T, int NT, int RT, int KS, int U>
__global__ __launch_bounds__(64 * KS) void dgrad_kernel(const T* __restrict__ WT, int N, const T* __restrict__ dG,
                                                        int nrow_tiles, int B, int BP, int G4,
                                                        float* __restrict__ out, int ld_out) {
  using M = Mma<T>;
  constexpr int VEC = M::VEC, KSTEP = 4 * VEC, NTILE = NT * RT, NPIECE = NTILE * 4, PPW = (NPIECE + KS - 1) / KS;
  extern __shared__ __attribute__((aligned(16))) unsigned char dgrad_smem[];
  float* red = reinterpret_cast<float*>(dgrad_smem);   // [KS][NTILE][4][64]
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), lane = threadIdx.x & 63;   // scalar: see wave_index note
  const int lrow = lane & 15, lq = lane >> 4;
  // Workgroups are handed to the 8 XCDs round-robin by their linear id.  As launched, an XCD would
  // own every 8th column group and see all of dG.  The id is re-mapped so that each XCD works
  // through a contiguous range of (row group, column group) pairs, column group fastest: the
  // workgroups that share a dG row group then share an L2, every XCD fetches only its own eighth
  // of dG, and the weight operand streams through each L2 once per round of resident workgroups
  // (measured: 136 -> 34 MB fetched per chunk on the 256 -> 1024 shape, 569 -> about 200 MB on
  // 512 -> 2048).
  const int gx = (int)gridDim.x, total = gx * (int)gridDim.y;
  const int id = (int)blockIdx.x + gx * (int)blockIdx.y;
  const int xcd = id & 7;
  const int work = xcd * (total >> 3) + min(xcd, total & 7) + (id >> 3);
  const int bx = work % gx, by = work / gx;
  const int ncol_tiles = (N + 15) / 16;
  const int nsteps = G4 / KSTEP;
  const T* abase[NT];
  const T* bbase[RT];
#pragma unroll
  for (int i = 0; i < NT; ++i)
    abase[i] = WT + ((size_t)min(bx * NT + i, ncol_tiles - 1) * nsteps * 64 + lane) * VEC;
#pragma unroll
  for (int j = 0; j < RT; ++j)
    bbase[j] = dG + ((size_t)min(by * RT + j, nrow_tiles - 1) * nsteps * 64 + lane) * VEC;
  f32x4 acc[NT][RT];
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int j = 0; j < RT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};
  for (int s0 = wave; s0 < nsteps; s0 += KS * U) {
    typename M::Frag af[U][NT], bf[U][RT];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      const size_t off = (size_t)min(s0 + u * KS, nsteps - 1) * 64 * VEC;
#pragma unroll
      for (int i = 0; i < NT; ++i) af[u][i] = M::load(abase[i] + off);
#pragma unroll
      for (int j = 0; j < RT; ++j) bf[u][j] = M::load(bbase[j] + off);
    }
#pragma unroll
    for (int u = 0; u < U; ++u)
      if (s0 + u * KS < nsteps) {
#pragma unroll
        for (int i = 0; i < NT; ++i)
#pragma unroll
          for (int j = 0; j < RT; ++j) acc[i][j] = M::mma(af[u][i], bf[u][j], acc[i][j]);
      }
  }
#pragma unroll
  for (int i = 0; i < NT; ++i)
#pragma unroll
    for (int j = 0; j < RT; ++j)
#pragma unroll
      for (int r = 0; r < 4; ++r) red[((wave * NTILE + i * RT + j) * 4 + r) * 64 + lane] = acc[i][j][r];
  __syncthreads();
#pragma unroll
  for (int q = 0; q < PPW; ++q) {
    const int piece = wave + q * KS;
    if (piece >= NPIECE) break;
    float v = 0.0f;
    for (int w = 0; w < KS; ++w) v += red[(w * NPIECE + piece) * 64 + lane];   // fixed order
    const int tile = piece >> 2, r = piece & 3;
    const int tn = tile / RT, tr = tile % RT;
    const int row = (by * RT + tr) * 16 + lrow;   // padded row: slot * BP + b
    const int n = (bx * NT + tn) * 16 + 4 * lq + r;
    const int slot = row / BP, b = row % BP;
    if (row >= nrow_tiles * 16 || b >= B || n >= N) continue;
    out[((size_t)slot * B + b) * ld_out + n] = v;
  }
}

template <class T, int NT, int RT, int KS, int U>
static hipError_t launch_dgrad_cfg(dim3 grid, const T* WT, int N, const T* dG, int nrow_tiles, const Dims& d, float* out,
                                   int ld_out, hipStream_t st) {
  const size_t lds = (size_t)KS * NT * RT * 4 * 64 * sizeof(float);
  static bool configured = false;   // per instantiation; needed above 64 KiB only, harmless below
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(dgrad_kernel<T, NT, RT, KS, U>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
    if (e != hipSuccess) return e;
    configured = true;
  }
  dgrad_kernel<T, NT, RT, KS, U><<<grid, dim3(64 * KS), lds, st>>>(WT, N, dG, nrow_tiles, d.B, d.BP, d.G4, out, ld_out);
  return hipGetLastError();
}

template <class T>
static hipError_t launch_dgrad_t(const Dims& d, const void* WT, int N, const void* dG, int nslots, float* out, int ld_out,
                                 hipStream_t st) {
  const int ncol_tiles = round_up(N, 16) / 16, nrow_tiles = nslots * d.BP / 16;
  // The largest output block per workgroup that still gives every compute unit one: each operand
  // byte a workgroup fetches is used for 64, 32 or 16 outputs.
  if (((ncol_tiles + 3) / 4) * ((nrow_tiles + 3) / 4) >= TARGET_WGS)
    return launch_dgrad_cfg<T, 4, 4, 8, 4>(dim3((ncol_tiles + 3) / 4, (nrow_tiles + 3) / 4), (const T*)WT, N, (const T*)dG,
                                           nrow_tiles, d, out, ld_out, st);
  if (((ncol_tiles + 1) / 2) * ((nrow_tiles + 3) / 4) >= TARGET_WGS)
    return launch_dgrad_cfg<T, 2, 4, 8, 4>(dim3((ncol_tiles + 1) / 2, (nrow_tiles + 3) / 4), (const T*)WT, N, (const T*)dG,
                                           nrow_tiles, d, out, ld_out, st);
  if (((ncol_tiles + 1) / 2) * ((nrow_tiles + 1) / 2) >= TARGET_WGS)
    return launch_dgrad_cfg<T, 2, 2, 8, 4>(dim3((ncol_tiles + 1) / 2, (nrow_tiles + 1) / 2), (const T*)WT, N, (const T*)dG,
                                           nrow_tiles, d, out, ld_out, st);
  return launch_dgrad_cfg<T, 1, 1, 8, 4>(dim3(ncol_tiles, nrow_tiles), (const T*)WT, N, (const T*)dG, nrow_tiles, d, out, ld_out,
                                         st);
}

hipError_t launch_dgrad_gemm(const Dims& d, const void* WT, int N, const void* dG, int nslots, float* out, int ld_out,
                             hipStream_t st) {
  return d.dtype ? launch_dgrad_t<__bf16>(d, WT, N, dG, nslots, out, ld_out, st)
                 : launch_dgrad_t<float>(d, WT, N, dG, nslots, out, ld_out, st);
}

// ---- time-batched GEMM on 256 x 256 workgroup tiles --------------------------------------------
// D[i][j] (+)= sum_k A[i][k] B[j][k] for the weight gradient over a chunk of steps (K = CH*B), used
// when dW has enough 256 x 256 tiles to fill the chip (the dx GEMM's output never has).  Both operands are fragment-tiled, so a 16-row tile of
// one macro step is a contiguous 1 KiB block.  A workgroup of 8 waves (2 along i, 4 along j) owns
// 256 x 256 outputs, each wave 128 x 64 (8 x 4 MFMA tiles, 128 accumulator registers); two waves
// share a SIMD, so one wave's LDS reads hide behind the other's MFMAs.  Per round of two macro
// steps (K = 64) the workgroup copies 32 + 32 operand fragments (64 KiB) from L2 into one of two
// LDS stages -- fetched into registers one round ahead -- and every wave reads the 8 + 4
// fragments per macro step it needs: each operand byte enters the compute unit once per
// workgroup, and there is one barrier per 64 of K.
// Workgroup ids are re-mapped so that the workgroups sharing an XCD (ids equal modulo 8) work
// through a contiguous range of (i-block, j-block) pairs, j fastest: they stream the same A panel
// through the L2 they share.
struct TgemmParams {
  const void* A;      // rows i: mt_total 16-row tiles, a_steps macro steps per tile
  const void* B;      // rows j
  int mt_total, nt_total, a_steps, b_steps;
  int nk;             // macro steps to contract over (from step 0)
  int gx, gy;         // workgroup grid: i-blocks, j-blocks
  float* acc;         // tile-ordered accumulator
  int accumulate;     // 0: overwrite it, 1: add to it
  // The first `full` workgroups (a multiple of the compute units) take one output block each over
  // the whole of K; the blocks left over, too few for a round of their own, are shared out `split`
  // ways along K so that the last round is short instead of mostly empty: part 0 adds into the
  // block's place in `acc`, part q > 0 into `extra` block (q - 1) * (gx * gy - full) + (block - full).
  // Which part sums what is fixed by the shape, so results do not depend on scheduling.
  int full, split;
  float* extra;
};

template <class T>
__global__ __launch_bounds__(512) void tgemm_kernel(TgemmParams p) {
  using M = Mma<T>;
  constexpr int VEC = M::VEC, FRAG = 64 * VEC;
  constexpr int TI = 8, TJ = 4;           // MFMA tiles per wave along i and j
  constexpr int WGT = 16;                 // 16-row tiles per workgroup along each axis
  typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
  extern __shared__ __attribute__((aligned(16))) unsigned char smem[];
  T* lds = reinterpret_cast<T*>(smem);    // [stage 2][macro step 2][16 tiles of A][FRAG]
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), lane = threadIdx.x & 63;   // scalar: see wave_index note
  const int wi = wave & 1, wj = wave >> 1;
  const int id = (int)blockIdx.x;
  int work, part = 0, nparts = 1;
  if (id < p.full) {
    const int xcd = id & 7;
    work = xcd * (p.full >> 3) + min(xcd, p.full & 7) + (id >> 3);
  } else {
    work = p.full + (id - p.full) / p.split;
    part = (id - p.full) % p.split;
    nparts = p.split;
  }
  const int bx = work / p.gy, by = work % p.gy;
  // this workgroup's share of K: rounds [r0, r1) of two macro steps each
  const int rounds_all = (p.nk + 1) >> 1;
  const int r0 = part * rounds_all / nparts, r1 = (part + 1) * rounds_all / nparts;
  const int nk = min(p.nk, 2 * r1) - 2 * r0;   // macro steps of the share (may be 0)
  const int nrounds = (nk + 1) >> 1;
  // a wave whose 128 x 64 outputs all lie outside the matrix (the last block of a ragged edge) only
  // helps to stage A
  const bool active = bx * WGT + wi * TI < p.mt_total && by * WGT + wj * TJ < p.nt_total;
  // A (the i operand, shared by the four waves of a row) goes L2 -> registers -> LDS: this wave
  // copies fragments f = wave*4 .. +4 of every round, f = ks * 16 + tile.  B (the j operand,
  // shared by two waves only) is fetched by each wave straight into its MFMA registers: LDS
  // carries 2/3 of the reads and half of the writes it would carry for both operands.
  const T* srcA[4];
  int ks_of[4];
#pragma unroll
  for (int q = 0; q < 4; ++q) {
    const int f = wave * 4 + q, ks = f >> 4, tile = f & 15;
    ks_of[q] = ks;
    srcA[q] = reinterpret_cast<const T*>(p.A) + ((size_t)min(bx * WGT + tile, p.mt_total - 1) * p.a_steps * 64 + lane) * VEC +
              (size_t)2 * r0 * FRAG;
  }
  const T* srcB[TJ];
#pragma unroll
  for (int j = 0; j < TJ; ++j)
    srcB[j] = reinterpret_cast<const T*>(p.B) + ((size_t)min(by * WGT + wj * TJ + j, p.nt_total - 1) * p.b_steps * 64 + lane) * VEC +
              (size_t)2 * r0 * FRAG;
  u32x4 ringA[2][4];
  typename M::Frag ringB[2][2][TJ];   // [set][macro step of the round][tile]
  auto fetch = [&](int set, int round) {
#pragma unroll
    for (int q = 0; q < 4; ++q) {
      const int s = min(round * 2 + ks_of[q], nk - 1);   // a macro step past the end is fetched (clamped) and never used
      ringA[set][q] = *reinterpret_cast<const u32x4*>(srcA[q] + (size_t)s * FRAG);
    }
    if (!active) return;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      const int s = min(round * 2 + ks, nk - 1);
#pragma unroll
      for (int j = 0; j < TJ; ++j) ringB[set][ks][j] = M::load(srcB[j] + (size_t)s * FRAG);
    }
  };
  auto stash = [&](int set, int stage) {
#pragma unroll
    for (int q = 0; q < 4; ++q)
      *reinterpret_cast<u32x4*>(&lds[((size_t)stage * 32 + wave * 4 + q) * FRAG + lane * VEC]) = ringA[set][q];
  };
  f32x4 acc[TI][TJ];
#pragma unroll
  for (int i = 0; i < TI; ++i)
#pragma unroll
    for (int j = 0; j < TJ; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  auto compute = [&](int r, int stage, int set) {
    if (!active) return;
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      if (r * 2 + ks < nk) {   // uniform
        const T* base = &lds[((size_t)stage * 32 + ks * 16) * FRAG + lane * VEC];
        // The wave's TI fragments of A come from LDS two ahead of the MFMAs that use them: two
        // reads, then TJ MFMAs and one more read in turn, so an LDS round trip always has eight
        // MFMAs to hide behind.  (Left to itself the scheduler puts every read right before its
        // MFMAs and waits for it.)  The group barriers fix that order for the instructions of
        // this block: 0x100 = LDS read, 0x008 = MFMA.
        typename M::Frag a[TI];
#pragma unroll
        for (int i = 0; i < TI; ++i) a[i] = M::load(base + (size_t)(wi * TI + i) * FRAG);
#pragma unroll
        for (int i = 0; i < TI; ++i)
#pragma unroll
          for (int j = 0; j < TJ; ++j) acc[i][j] = M::mma(a[i], ringB[set][ks][j], acc[i][j]);
        __builtin_amdgcn_sched_group_barrier(0x100, 2, 0);
#pragma unroll
        for (int i = 0; i < TI - 2; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, TJ, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 2 * TJ, 0);
      }
    }
  };

  if (nrounds > 0) {
    // Register set r & 1 holds round r: its A part is moved to LDS stage r & 1 one round early, its
    // B part is consumed in place; the set is refilled with round r + 2 once round r is computed.
    fetch(0, 0);
    fetch(1, 1);           // clamped when there is a single round
    stash(0, 0);
    __syncthreads();
    for (int r = 0; r < nrounds; r += 2) {   // unrolled by two so that sets and stages are static
      if (r + 1 < nrounds) stash(1, 1);
      compute(r, 0, 0);
      fetch(0, r + 2);
      __syncthreads();
      if (r + 1 < nrounds) {
        if (r + 2 < nrounds) stash(0, 0);
        compute(r + 1, 1, 1);
        fetch(1, r + 3);
        __syncthreads();
      }
    }
  }

  // Running sum in a tile-ordered accumulator: a wave's 32 tiles are one contiguous run and a
  // lane's four rows one float4, so the read-modify-write of every chunk is fully coalesced;
  // wgrad_finish_kernel converts it to the caller's row-major dW once at the end of the run.
  if (!active) return;   // nobody reads blocks outside the matrix
  const size_t block = part == 0 ? (size_t)work : (size_t)(part - 1) * (p.gx * p.gy - p.full) + (work - p.full);
  float4* accp = reinterpret_cast<float4*>(part == 0 ? p.acc : p.extra) + ((block * 8 + wave) * (TI * TJ)) * 64 + lane;
#pragma unroll
  for (int half = 0; half < 2; ++half) {   // two batches of 16 tiles: the old values pass through few registers
    float4 old[TI * TJ / 2];
    if (p.accumulate) {
#pragma unroll
      for (int q = 0; q < TI * TJ / 2; ++q) old[q] = accp[(size_t)(half * (TI * TJ / 2) + q) * 64];
    }
#pragma unroll
    for (int q = 0; q < TI * TJ / 2; ++q) {
      const int t = half * (TI * TJ / 2) + q;
      f32x4 v = acc[t / TJ][t % TJ];
      if (p.accumulate) {
        v[0] += old[q].x;
        v[1] += old[q].y;
        v[2] += old[q].z;
        v[3] += old[q].w;
      }
      accp[(size_t)t * 64] = float4{v[0], v[1], v[2], v[3]};
    }
  }
}

constexpr int TGEMM_LDS_BYTES = 2 * 32 * 1024;
constexpr int TGEMM_MIN_TILES = 192;   // below this the output does not fill the chip with 256 x 256 tiles

template <class T>
static hipError_t launch_tgemm(const TgemmParams& p, hipStream_t st) {
  static bool configured = false;
  if (!configured) {
    hipError_t e = hipFuncSetAttribute(reinterpret_cast<const void*>(tgemm_kernel<T>),
                                       hipFuncAttributeMaxDynamicSharedMemorySize, TGEMM_LDS_BYTES);
    if (e != hipSuccess) return e;
    configured = true;
  }
  tgemm_kernel<T><<<dim3(p.full + (p.gx * p.gy - p.full) * p.split), dim3(512), TGEMM_LDS_BYTES, st>>>(p);
  return hipGetLastError();
}

// How the 256 x 256 output blocks are dealt out: whole rounds of one block per compute unit over all
// of K, and the blocks left over split along K as many ways as fit one more round (at most four).
constexpr int TGEMM_ROUND = 256;
static void tgemm_shares(int blocks, int& full, int& split) {
  full = blocks / TGEMM_ROUND * TGEMM_ROUND;
  const int rest = blocks - full;
  split = rest == 0 ? 1 : std::max(1, std::min(4, TGEMM_ROUND / rest));
  if (split == 1) full = blocks;
}

// ---- dx GEMM on the 256 x 256 blocks ---------------------------------------------------------
// dx[(step, b)][n] = sum_k dG[(step, b)][k] W_ih^T[n][k] over a chunk of steps has few output blocks
// (cfg3: 2 x 16) and a long K = 4H, so every block's K is shared out over `split` workgroups, each
// writing its partial block; dx_finish_kernel adds the parts in a fixed order and stores the rows
// of real sequences.  The partial blocks live in a scratch buffer the caller lends (the chunk's
// dG^T buffer, which nobody reads between this chunk's dW GEMM and the next chunk that fills it).
// Used when that gives the chip at least 192 workgroups with at least 16 macro steps each.
constexpr int DX_MAX_SPLIT = 8;
struct DxBlocks {
  int gx, gy, split;   // blocks along n, along the rows of a full chunk, K shares per block (0: not used)
};
static DxBlocks dx_blocks(const Dims& d, size_t scratch_bytes) {
  DxBlocks b{0, 0, 0};
  if (!d.dtype || d.NX < 256) return b;
  b.gx = (d.NX / 16 + 15) / 16;
  b.gy = (d.CH * d.BP / 16 + 15) / 16;
  const int blocks = b.gx * b.gy, nk = d.G4 / 32;
  const size_t fit = scratch_bytes / ((size_t)blocks * 256 * 256 * sizeof(float));
  const int split = (int)std::min<size_t>(std::min(DX_MAX_SPLIT, std::min(TGEMM_ROUND / blocks, nk / 16)), fit);
  if (split >= 1 && blocks * split >= 192) b.split = split;
  return b;
}

// partial[part][block][wave][tile][lane] (tgemm_kernel's accumulator order) -> dx rows.  One thread
// per float4 of a block: four consecutive n of one (step, b) row.
__global__ void dx_finish_kernel(const float4* __restrict__ partial, int blocks, int split, int gy, int nrows, int B, int BP,
                                 int I, float* __restrict__ out, int ld_out) {
  const size_t total = (size_t)blocks * (256 * 256 / 4), stride = (size_t)gridDim.x * blockDim.x;
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
    const int lane = (int)(idx & 63), tile = (int)((idx >> 6) & 31), wave = (int)((idx >> 11) & 7);
    const int block = (int)(idx >> 14);
    const int bx = block / gy, by = block % gy;
    const int wi = wave & 1, wj = wave >> 1, ti = tile >> 2, tj = tile & 3;
    const int n = ((bx * 16 + wi * 8 + ti) * 16) + 4 * (lane >> 4);
    const int row = ((by * 16 + wj * 4 + tj) * 16) + (lane & 15);   // padded row: slot * BP + b
    const int slot = row / BP, b = row % BP;
    if (row >= nrows || b >= B || n >= I) continue;
    float4 u[DX_MAX_SPLIT];   // all parts fetched before the first addition: the loads overlap
#pragma unroll
    for (int q = 0; q < DX_MAX_SPLIT; ++q)
      if (q < split) u[q] = partial[(size_t)q * total + idx];
    float4 v = u[0];
#pragma unroll
    for (int q = 1; q < DX_MAX_SPLIT; ++q)   // fixed order
      if (q < split) {
        v.x += u[q].x;
        v.y += u[q].y;
        v.z += u[q].z;
        v.w += u[q].w;
      }
    float* dst = out + ((size_t)slot * B + b) * ld_out + n;
    if (n + 3 < I && (ld_out & 3) == 0) {
      *reinterpret_cast<float4*>(dst) = v;
    } else {
      const float e[4] = {v.x, v.y, v.z, v.w};
      for (int r = 0; r < 4 && n + r < I; ++r) dst[r] = e[r];
    }
  }
}

bool dx_gemm_uses_blocks(const Dims& d, size_t scratch_bytes) { return dx_blocks(d, scratch_bytes).split > 0; }

hipError_t launch_dx_gemm(const Dims& d, const void* WTx, const void* dG, int nslots, float* dx, void* scratch,
                          size_t scratch_bytes, hipStream_t st) {
  const DxBlocks b = dx_blocks(d, scratch_bytes);
  if (b.split == 0) return launch_dgrad_gemm(d, WTx, d.I, dG, nslots, dx, d.I, st);
  TgemmParams p{};
  p.A = WTx;
  p.B = dG;
  p.mt_total = d.NX / 16;
  p.nt_total = nslots * d.BP / 16;
  p.a_steps = p.b_steps = d.G4 / 32;
  p.nk = d.G4 / 32;
  p.gx = b.gx;
  p.gy = (p.nt_total + 15) / 16;   // a short chunk has fewer blocks; the shares stay those of the shape
  p.acc = reinterpret_cast<float*>(scratch);
  p.accumulate = 0;
  p.full = 0;
  p.split = b.split;
  p.extra = p.acc + (size_t)p.gx * p.gy * 256 * 256;
  hipError_t e = launch_tgemm<__bf16>(p, st);
  if (e != hipSuccess) return e;
  const int blocks = p.gx * p.gy;
  dx_finish_kernel<<<dim3(std::min(blocks * 64, 4096)), dim3(256), 0, st>>>(reinterpret_cast<const float4*>(scratch), blocks, b.split,
                                                                           p.gy, nslots * d.BP, d.B, d.BP, d.I, dx, d.I);
  return hipGetLastError();
}

// The weight gradient runs on the 256 x 256 tiles when the operands are bf16 and dW has enough tiles.
static bool wgrad_uses_big_tiles(const Dims& d) {
  if (!d.dtype) return false;
  const int gx = (d.G4 / 16 + 15) / 16, gy = (d.NA / 16 + 15) / 16;
  return gx * gy >= TGEMM_MIN_TILES;
}

// ---- x transposed into the weight-gradient operand ----------------------------------------------

template <class T>
__global__ void transpose_x_kernel(const float* __restrict__ x, int rows, int I, int KC, int ones_row,
                                   T* __restrict__ aT) {
  // x: [rows][I] (rows = nslots*B consecutive (step, b) pairs) -> aT[i][row]; the first column of
  // blocks also sets aT[ones_row][row] = 1, the operand row that turns db into a column of dW.
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
    if (i < I && r < rows) aT[ft_offset<T>(i, r, KC / (4 * Mma<T>::VEC))] = (T)tile[tx][ii];
  }
  if (blockIdx.y == 0 && ty == 0 && r0 + tx < rows) aT[ft_offset<T>(ones_row, r0 + tx, KC / (4 * Mma<T>::VEC))] = (T)1.0f;
}

hipError_t launch_transpose_x(const Dims& d, const float* x_first, int nslots, void* aT, hipStream_t st) {
  const int rows = nslots * d.B;
  dim3 grid((rows + 31) / 32, (d.I + 31) / 32), block(256);
  if (d.dtype)
    transpose_x_kernel<__bf16><<<grid, block, 0, st>>>(x_first, rows, d.I, d.KC, d.NX + d.HP, (__bf16*)aT);
  else
    transpose_x_kernel<float><<<grid, block, 0, st>>>(x_first, rows, d.I, d.KC, d.NX + d.HP, (float*)aT);
  return hipGetLastError();
}

// Zeroes columns [c0, c1) of the two weight-gradient operands (dGT: G4 rows, aT: NA rows).
template <class T>
__global__ void zero_operand_columns_kernel(T* __restrict__ dGT, int G4, T* __restrict__ aT, int NA, int KC, int c0, int c1) {
  const int ncols = c1 - c0, ncs = KC / (4 * Mma<T>::VEC);
  const size_t total = (size_t)(G4 + NA) * ncols;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t i = (size_t)blockIdx.x * blockDim.x + threadIdx.x; i < total; i += stride) {
    const int row = (int)(i / ncols), col = c0 + (int)(i % ncols);
    if (row < G4)
      dGT[ft_offset<T>(row, col, ncs)] = (T)0.0f;
    else
      aT[ft_offset<T>(row - G4, col, ncs)] = (T)0.0f;
  }
}

hipError_t launch_zero_operand_columns(const Dims& d, void* dGT, void* aT, int c0, int c1, hipStream_t st) {
  if (c1 <= c0) return hipSuccess;
  if (c0 < 0 || c1 > d.KC) return hipErrorInvalidValue;
  const size_t total = (size_t)(d.G4 + d.NA) * (c1 - c0);
  size_t blocks = (total + 255) / 256;
  if (blocks > 2048) blocks = 2048;
  if (d.dtype)
    zero_operand_columns_kernel<__bf16><<<dim3((unsigned)blocks), dim3(256), 0, st>>>((__bf16*)dGT, d.G4, (__bf16*)aT, d.NA, d.KC, c0, c1);
  else
    zero_operand_columns_kernel<float><<<dim3((unsigned)blocks), dim3(256), 0, st>>>((float*)dGT, d.G4, (float*)aT, d.NA, d.KC, c0, c1);
  return hipGetLastError();
}

// ---- weight-gradient GEMM: dW[row(m)][n] (+)= sum_k dGT[m][k] * aT[n][k] ------------------------

// A workgroup of 2 x 2 waves owns a block of 2*WT x 2*WT MFMA tiles of dW (128 x 128 elements for
// WT = 4, 64 x 64 for WT = 2, used when the larger block would leave most compute units idle);
// each wave a WT x WT quarter.  Per macro step the workgroup copies the 2*WT + 2*WT operand
// fragments of its block (1 KiB each, already in fragment order) from HBM/L2 into LDS with fully
// coalesced 16-byte loads -- fetched PD macro steps ahead through a ring of registers -- and every
// wave reads the WT + WT fragments it needs from LDS, so each operand byte crosses the L2 fabric
// once per workgroup instead of once per wave.  gridDim.z workgroups may share one output block,
// each with its own part of K and its own partial accumulator.
template <class T, int WT>
__global__ __launch_bounds__(256) void wgrad_kernel(const T* __restrict__ dGT, const T* __restrict__ aT, int K, int KC,
                                                    int G4, int NTOT, int accumulate, float* __restrict__ dWacc) {
  using M = Mma<T>;
  constexpr int VEC = M::VEC, KSTEP = 4 * VEC, PD = 3;
  constexpr int FRAG = 64 * VEC;                  // elements of one fragment block (1 KiB)
  typedef __attribute__((ext_vector_type(4))) unsigned int u32x4;
  __shared__ __attribute__((aligned(16))) T lds[2][4 * WT * FRAG];
  const int wave = __builtin_amdgcn_readfirstlane((int)(threadIdx.x >> 6)), lane = threadIdx.x & 63;   // scalar: see wave_index note
  const int wm = wave & 1, wn = wave >> 1;
  const int MT = G4 / 16, NT = NTOT / 16;
  const int mt_wg = blockIdx.x * 2 * WT, nt_wg = blockIdx.y * 2 * WT;
  const int ncs = KC / KSTEP;    // macro steps per row tile in the fragment-tiled operands
  // gridDim.z workgroups share one output tile, each taking a contiguous part of the macro steps
  // that hold data and keeping its own partial accumulator (summed, in a fixed order, by
  // wgrad_finish_kernel).  A part may be empty (short last chunk): it then only initialises or
  // keeps its partial sum.
  const int nk_all = K / KSTEP;
  const int k_begin = (int)((long long)nk_all * blockIdx.z / gridDim.z);
  const int nk = (int)((long long)nk_all * (blockIdx.z + 1) / gridDim.z) - k_begin;
  // this thread copies blocks q*4 + wave, q = 0..WT-1: the first 2*WT blocks are dGT row tiles,
  // the other 2*WT are aT row tiles
  const T* src[WT];
#pragma unroll
  for (int q = 0; q < WT; ++q) {
    const int blk = q * 4 + wave;
    if (blk < 2 * WT)
      src[q] = dGT + (((size_t)min(mt_wg + blk, MT - 1) * ncs + k_begin) * 64 + lane) * VEC;
    else
      src[q] = aT + (((size_t)min(nt_wg + blk - 2 * WT, NT - 1) * ncs + k_begin) * 64 + lane) * VEC;
  }
  u32x4 ring[PD][WT];
  auto fetch = [&](int stage, int ks) {
    const size_t off = (size_t)min(ks, nk - 1) * FRAG;
#pragma unroll
    for (int q = 0; q < WT; ++q) ring[stage][q] = *reinterpret_cast<const u32x4*>(src[q] + off);
  };
  auto stash = [&](int stage, int buf) {
#pragma unroll
    for (int q = 0; q < WT; ++q)
      *reinterpret_cast<u32x4*>(&lds[buf][(q * 4 + wave) * FRAG + lane * VEC]) = ring[stage][q];
  };
  f32x4 acc[WT][WT];
#pragma unroll
  for (int i = 0; i < WT; ++i)
#pragma unroll
    for (int j = 0; j < WT; ++j) acc[i][j] = f32x4{0.f, 0.f, 0.f, 0.f};

  if (nk > 0) {   // uniform over the workgroup
#pragma unroll
  for (int st = 0; st < PD; ++st) fetch(st, st);
  stash(0, 0);
  __syncthreads();
  for (int k0 = 0; k0 < nk; k0 += PD) {
#pragma unroll
    for (int j = 0; j < PD; ++j) {
      const int ks = k0 + j;           // macro step computed now (held in lds[ks & 1])
      if (ks < nk) {
        fetch(j, ks + PD);             // ring slot j was stashed for step ks; refill it PD steps ahead
        typename M::Frag af[WT], bf[WT];
#pragma unroll
        for (int i = 0; i < WT; ++i) bf[i] = M::load(&lds[ks & 1][(2 * WT + wn * WT + i) * FRAG + lane * VEC]);
#pragma unroll
        for (int i = 0; i < WT; ++i) af[i] = M::load(&lds[ks & 1][(wm * WT + i) * FRAG + lane * VEC]);
#pragma unroll
        for (int i = 0; i < WT; ++i)
#pragma unroll
          for (int jj = 0; jj < WT; ++jj) acc[i][jj] = M::mma(af[i], bf[jj], acc[i][jj]);
        // order of this block's LDS reads (0x100) and MFMAs (0x008): what the first row of MFMAs
        // needs (af[0] and every bf) plus af[1], then a row of MFMAs and the next af in turn, so
        // that only the first reads of a macro step are waited for
        __builtin_amdgcn_sched_group_barrier(0x100, WT + 2, 0);
#pragma unroll
        for (int i = 0; i < WT - 2; ++i) {
          __builtin_amdgcn_sched_group_barrier(0x008, WT, 0);
          __builtin_amdgcn_sched_group_barrier(0x100, 1, 0);
        }
        __builtin_amdgcn_sched_group_barrier(0x008, 2 * WT, 0);
        if (ks + 1 < nk) stash((j + 1) % PD, (ks + 1) & 1);
      }
      __syncthreads();
    }
  }
  }

  // Epilogue: the running sum lives in a tile-ordered accumulator (each wave's quarter is one
  // contiguous run, a lane's four accumulator rows one float4), so the
  // read-modify-write of every chunk is fully coalesced; wgrad_finish_kernel converts it to the
  // caller's row-major dW once at the end of the run.
  float4* accp = reinterpret_cast<float4*>(dWacc) +
                 (((size_t)blockIdx.z * gridDim.x * gridDim.y + blockIdx.x * gridDim.y + blockIdx.y) * 4 + wave) * (WT * WT) * 64 + lane;
  if (accumulate) {
    float4 old[WT * WT];
#pragma unroll
    for (int q = 0; q < WT * WT; ++q) old[q] = accp[q * 64];
#pragma unroll
    for (int q = 0; q < WT * WT; ++q) {
      acc[q / WT][q % WT][0] += old[q].x;
      acc[q / WT][q % WT][1] += old[q].y;
      acc[q / WT][q % WT][2] += old[q].z;
      acc[q / WT][q % WT][3] += old[q].w;
    }
  }
#pragma unroll
  for (int q = 0; q < WT * WT; ++q)
    accp[q * 64] = float4{acc[q / WT][q % WT][0], acc[q / WT][q % WT][1], acc[q / WT][q % WT][2], acc[q / WT][q % WT][3]};
}

// dW_ih[row][n] / dW_hh[row][n] <- the tile-ordered accumulator (see wgrad_kernel's epilogue).
// The accumulator's column NX + HP (operand row of ones) holds the bias gradient.  ngates = 4
// (LSTM: db [4H]) or 3 (GRU: db = [db_ih | db_hh], 6H); the packed row of a gate block differs
// between the input and the recurrent side for the GRU (packed_gate_x / packed_gate_h).
__global__ void wgrad_finish_kernel(const float* __restrict__ dWacc, int WT, int grid_y, int nsplit, size_t split_stride,
                                    int NX, int HP, int I, int H, int cell, float* __restrict__ dW_ih,
                                    float* __restrict__ dW_hh, float* __restrict__ db, int blocks) {
  const int ngates = cell ? 3 : 4;
  const size_t nih = (size_t)ngates * H * I, nhh = (size_t)ngates * H * H, nb = (size_t)(cell ? 6 : 4) * H;
  const size_t total = nih + nhh + nb;
  const size_t stride = (size_t)gridDim.x * blockDim.x;
  for (size_t idx = (size_t)blockIdx.x * blockDim.x + threadIdx.x; idx < total; idx += stride) {
    int row, np;
    bool recurrent;
    float* dst;
    if (idx < nih) {
      row = (int)(idx / I);
      np = (int)(idx % I);
      recurrent = false;
      dst = dW_ih + idx;
    } else if (idx < nih + nhh) {
      const size_t j = idx - nih;
      row = (int)(j / H);
      np = NX + (int)(j % H);
      recurrent = true;
      dst = dW_hh + j;
    } else {
      row = (int)(idx - nih - nhh);
      recurrent = row >= ngates * H;   // only the GRU has a second (recurrent) bias block
      if (recurrent) row -= ngates * H;
      np = NX + HP;
      dst = db + (idx - nih - nhh);
    }
    const int gate = row / H, u = row % H;
    int prow = gate;                                    // packed row of this gate block
    if (cell) prow = recurrent ? (gate == 2 ? 3 : gate) : gate;
    const int mp = 4 * u + prow;
    const int mt = mp >> 4, lq = (mp & 15) >> 2, r = mp & 3;
    const int nt = np >> 4, lrow = np & 15;
    size_t off;
    if (WT == 0) {   // tgemm_kernel's blocks: 2 x 4 waves of 8 x 4 tiles per 256 x 256 workgroup
      const int wgx = mt >> 4, wi = (mt & 15) >> 3, ti = mt & 7;
      const int wgy = nt >> 4, wj = (nt & 15) >> 2, tj = nt & 3;
      const size_t inner = (((size_t)(wi + 2 * wj) * 32 + (ti * 4 + tj)) * 64 + (lq * 16 + lrow)) * 4 + r;
      const int block = wgx * grid_y + wgy, first_shared = (int)split_stride;
      constexpr size_t BLOCK = 256 * 256;
      float v = dWacc[(size_t)block * BLOCK + inner];
      if (block >= first_shared)   // a block whose K was shared out: the other parts' sums, fixed order
        for (int sp = 1; sp < nsplit; ++sp)
          v += dWacc[((size_t)blocks + (size_t)(sp - 1) * (blocks - first_shared) + (block - first_shared)) * BLOCK + inner];
      *dst = v;
      continue;
    } else {
      const int wgx = mt / (2 * WT), wm = (mt % (2 * WT)) / WT, i = mt % WT;
      const int wgy = nt / (2 * WT), wn = (nt % (2 * WT)) / WT, jj = nt % WT;
      off = ((((size_t)(wgx * grid_y + wgy) * 4 + (wm + 2 * wn)) * (WT * WT) + (i * WT + jj)) * 64 + (lq * 16 + lrow)) * 4 + r;
    }
    float v = dWacc[off];
    for (int sp = 1; sp < nsplit; ++sp) v += dWacc[(size_t)sp * split_stride + off];   // partial sums, fixed order
    *dst = v;
  }
}

// Wave tile of the weight-gradient GEMM (4 x 4 MFMA tiles, 128 x 128 per workgroup, whenever the
// output has at least one such tile in each direction; else 2 x 2) and the number of workgroups
// that split K for one output tile: enough to give the chip about 1.5 workgroups per compute unit
// when the output alone has too few tiles (long chunks of small matrices).
static int wgrad_wave_tile(const Dims& d) {
  const int MT = d.G4 / 16, NT = d.NA / 16;
  return (MT >= 8 && NT >= 8) ? 4 : 2;
}
static int wgrad_splits(const Dims& d) {
  const int WT = wgrad_wave_tile(d);
  const int tiles = ((d.G4 / 16 + 2 * WT - 1) / (2 * WT)) * ((d.NA / 16 + 2 * WT - 1) / (2 * WT));
  const int s = (384 + tiles / 2) / tiles;
  return s < 1 ? 1 : (s > 8 ? 8 : s);
}
static size_t wgrad_partial_floats(const Dims& d) {   // one partial accumulator
  const int WT = wgrad_wave_tile(d);
  const size_t gx = (d.G4 / 16 + 2 * WT - 1) / (2 * WT), gy = (d.NA / 16 + 2 * WT - 1) / (2 * WT);
  return gx * gy * 4 * WT * WT * 64 * 4;
}

size_t wgrad_accumulator_bytes(const Dims& d) {
  if (wgrad_uses_big_tiles(d)) {   // one padded 256 x 256 block per workgroup
    const size_t gx = (d.G4 / 16 + 15) / 16, gy = (d.NA / 16 + 15) / 16;
    int full, split;
    tgemm_shares((int)(gx * gy), full, split);
    return (gx * gy + (gx * gy - full) * (split - 1)) * 256 * 256 * sizeof(float);
  }
  return wgrad_partial_floats(d) * wgrad_splits(d) * sizeof(float);
}

template <class T>
static void launch_wgrad_t(const Dims& d, const void* dGT, const void* aT, int K, int accumulate, float* dWacc,
                           hipStream_t st) {
  const int NTOT = d.NA, WT = wgrad_wave_tile(d);
  dim3 grid((d.G4 / 16 + 2 * WT - 1) / (2 * WT), (NTOT / 16 + 2 * WT - 1) / (2 * WT), wgrad_splits(d)), block(256);
  if (WT == 4)
    wgrad_kernel<T, 4><<<grid, block, 0, st>>>((const T*)dGT, (const T*)aT, K, d.KC, d.G4, NTOT, accumulate, dWacc);
  else
    wgrad_kernel<T, 2><<<grid, block, 0, st>>>((const T*)dGT, (const T*)aT, K, d.KC, d.G4, NTOT, accumulate, dWacc);
}

hipError_t launch_wgrad(const Dims& d, const void* dGT, const void* aT, int nslots, int accumulate, float* dWacc,
                        hipStream_t st) {
  const int kstep = d.dtype ? 32 : 16;
  const int K = round_up(nslots * d.B, kstep);   // columns past nslots*B are zero
  if (wgrad_uses_big_tiles(d)) {
    TgemmParams p{};
    p.A = dGT;
    p.B = aT;
    p.mt_total = d.G4 / 16;
    p.nt_total = d.NA / 16;
    p.a_steps = p.b_steps = d.KC / 32;
    p.nk = K / 32;
    p.gx = (p.mt_total + 15) / 16;
    p.gy = (p.nt_total + 15) / 16;
    p.acc = dWacc;
    p.accumulate = accumulate;
    tgemm_shares(p.gx * p.gy, p.full, p.split);
    p.extra = dWacc + (size_t)p.gx * p.gy * 256 * 256;
    return launch_tgemm<__bf16>(p, st);
  }
  if (d.dtype)
    launch_wgrad_t<__bf16>(d, dGT, aT, K, accumulate, dWacc, st);
  else
    launch_wgrad_t<float>(d, dGT, aT, K, accumulate, dWacc, st);
  return hipGetLastError();
}

hipError_t launch_wgrad_finish(const Dims& d, const float* dWacc, float* dW_ih, float* dW_hh, float* db,
                               hipStream_t st) {
  if (wgrad_uses_big_tiles(d)) {
    const int gx = (d.G4 / 16 + 15) / 16, gy = (d.NA / 16 + 15) / 16;
    int full, split;
    tgemm_shares(gx * gy, full, split);
    // nsplit and split_stride: here the shares of the left-over blocks and the first of those blocks
    wgrad_finish_kernel<<<dim3(2048), dim3(256), 0, st>>>(dWacc, 0, gy, split, (size_t)full, d.NX, d.HP, d.I, d.H, d.cell,
                                                          dW_ih, dW_hh, db, gx * gy);
    return hipGetLastError();
  }
  const int WT = wgrad_wave_tile(d);
  const int grid_y = (d.NA / 16 + 2 * WT - 1) / (2 * WT);
  wgrad_finish_kernel<<<dim3(2048), dim3(256), 0, st>>>(dWacc, WT, grid_y, wgrad_splits(d), wgrad_partial_floats(d), d.NX, d.HP,
                                                        d.I, d.H, d.cell, dW_ih, dW_hh, db, 0);
  return hipGetLastError();
}

}  // namespace mebptt
