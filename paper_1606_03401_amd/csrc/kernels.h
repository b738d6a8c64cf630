// Launch wrappers for the HIP kernels (defined in kernels.hip).  Not part of the ABI.
//
// Shapes and padded operand layouts (all chosen so that every vector load of a GEMM operand is
// 16-byte aligned and in bounds; padding is zero):
//   HP = H rounded up to 16 (32 for bf16 operands),  KX = I rounded up to 32,  KH = H rounded up to 32,
//   KP = KX + KH,
//   NX = I rounded up to 16,  BP = B rounded up to 16,  G4 = 4 * HP.
// The logical matrices below are all stored fragment-tiled (16-row tiles, one contiguous 1 KiB
// block per tile and macro step; the exact index map is next to ft_offset in kernels.hip):
//   Wp  [G4][KP]         forward operand: row 4*u + gate is row gate*H + u of [W_ih | W_hh];
//                        columns [0,KX) hold W_ih, [KX,KP) hold W_hh.  (GRU: the four rows of a
//                        unit are r, z, n_x = [W_in | 0], n_h = [0 | W_hn]; see packed_gate_x/h.)
//   WTh [HP][G4]         WTh[n][4u+gate] = W_hh[gate*H+u][n]  (operand of dh_{s-1} = dG_s W_hh)
//   WTx [NX][G4]         WTx[n][4u+gate] = W_ih[gate*H+u][n]  (operand of dx_s   = dG_s W_ih)
//   dG  [CH*BP][G4]      gate pre-activation gradients of one chunk of CH consecutive steps, row
//                        slot*BP + b, columns in the permuted order 4u + gate; slot = (step-1) % CH.
//   dGT [G4][KC]         the same values transposed, KC = CH*B rounded up to 32, column
//                        slot*B + b: operand of the weight-gradient GEMM.
//   aT  [NA][KC]         NA = NX+HP+16.  Rows [0,NX): x_s transposed; rows [NX,NX+HP): h_{s-1}
//                        transposed; row NX+HP: ones (its dW column is db); the rest zero.
// Plain arrays:
//   bp  [G4] fp32        bias in the permuted order: bp[4u + gate] = b[gate*H + u].
//
// State units.  A unit (the granule of the slot pool) holds a hidden state (h, c) or a pair of gate
// planes (GRU: (h, n_h pre-activation) and the pairs (r, z), (n, unused)); it is `unit` floats long (a multiple of 64).  Gate planes and c are plain [B][H] fp32.
// The h plane comes first in its unit and is `hplane` floats long:
//   fp32 operands: plain [B][H] fp32.
//   bf16 operands: the SAME 4 bytes per element, split into two fragment-tiled 16-bit planes of
//     the logical matrix [BP][KH]: `hi` = the value rounded to bf16 (half-up), ready to be fetched
//     as a GEMM operand in 1 KiB blocks, then `lo` = the low 16 bits of the fp32 pattern.  The fp32
//     value is recovered exactly as ((hi - (lo >> 15)) << 16) | lo.
// OpT is float (gemm_dtype 0) or bf16 (gemm_dtype 1); accumulation is always fp32.
#pragma once

#include <hip/hip_runtime.h>

#include <cstddef>
#include <cstdint>

namespace mebptt {

struct Dims {
  int B, I, H;
  int HP, KX, KH, KP, NX, BP, G4, NA;
  int CH, KC;   // steps per weight-gradient chunk, padded K of that GEMM
  int dtype;    // 0 fp32, 1 bf16
  int cell;     // 0 LSTM, 1 GRU
  size_t hplane, unit;   // floats: the h part of a hidden-state unit, a whole unit
  size_t op_bytes() const { return dtype ? 2 : 4; }
};

inline int round_up(int v, int m) { return (v + m - 1) / m * m; }

Dims make_dims(int B, int I, int H, int dtype, int cell);

hipError_t launch_fill_zero(void* p, size_t bytes, hipStream_t st);
hipError_t launch_prep_weights(const Dims& d, const float* W_ih, const float* W_hh, const float* b, void* Wp,
                               float* bp, void* WTh, void* WTx, hipStream_t st);
// dst unit <- (h0, c0), NULL meaning zeros.
hipError_t launch_init_state(const Dims& d, const float* h0, const float* c0, float* dst_unit, hipStream_t st);

// One forward operation: reads x_s [B,I] and the hidden state at src; writes (h,c) to dst and,
// when gates != NULL, (i,f) and (g,o) to the two units starting at `gates`.
hipError_t launch_forward(const Dims& d, const void* Wp, const float* bp, const float* x_s, const float* src_unit,
                          float* dst_unit, float* gates_units, hipStream_t st);

// n independent forward operations in one launch (n <= forward_batch_max_steps()): operation j reads
// x[j] and the hidden-state unit src[j] and writes the state and the gates to the three units at
// dst[j].  Same bits as launch_forward.  bf16 LSTM only (can_run_forward_batch).
int forward_batch_max_steps();
bool can_run_forward_batch(const Dims& d);
hipError_t launch_forward_batch(const Dims& d, const void* Wp, const float* bp, int n, const float* const* x,
                                const float* const* src, float* const* dst, hipStream_t st);

struct BackwardArgs {
  const void* WTh;
  const void* dG_next;    // dG rows of step s+1 (BP rows of the chunk buffer), or NULL for s = t
  const float* state;     // unit (h_s, c_s); the gates follow in the next two units
  const float* prev;      // unit (h_{s-1}, c_{s-1})
  const float* dy_s;      // [B,H] or NULL
  int dy_is_h;            // built-in loss: the injected gradient is h_s itself
  float* dc;              // [B,H] running gradient w.r.t. the cell state, updated in place
  void* dG_cur;           // dG rows of step s (written)
  void* dGT;              // chunk-transposed copy (written at column col0 + b)
  void* aT;               // h_{s-1} transposed goes to rows [NX, NX+HP) at column col0 + b
  int col0;               // slot * B
  float* y_out_s;         // [B,H] or NULL
};
// One backward operation (the sequential half): dh_s = dG_{s+1} W_hh + dy_s, then the pointwise
// LSTM backward producing dG_s and dc_{s-1}.
hipError_t launch_backward(const Dims& d, const BackwardArgs& a, hipStream_t st);

// Measurement: a kernel with the grid of the forward launch of this shape whose workgroups only
// read the operand panels their forward counterparts read (weights from Wp, activations from
// `act`, act_bytes of readable memory); *delivered_bytes = what all workgroups read together.
hipError_t launch_forward_stream(const Dims& d, const void* Wp, const void* act, size_t act_bytes, float* sink,
                                 size_t* delivered_bytes, hipStream_t st);

// True when the shape runs the large-K kernel configurations, for which a backward step and an
// independent forward step can share one launch.
bool can_fuse_pair(const Dims& d);
// One launch carrying the backward step `a` and one forward operation (arguments as
// launch_forward).  The caller guarantees the forward step writes nothing the backward step reads.
hipError_t launch_backward_forward_pair(const Dims& d, const BackwardArgs& a, const void* Wp, const float* bp,
                                        const float* x_s, const float* src_unit, float* dst_unit, float* gates_units,
                                        hipStream_t st);

// A chain of consecutive forward operations in one launch, with the gate weights resident on the
// chip (shapes for which can_run_forward_chain() holds).  Step j (0-based) of the chain consumes
// x_first + j*B*I; its state goes to steps[j].out and its gates to the two units at
// steps[j].gates where these are not NULL (states nobody asked for never leave the chip).
// `ring` (forward_chain_ring_bytes) and `sync` (forward_chain_sync_bytes, zero before the first
// launch of a run) are workspace; `base` is the number of arrivals earlier launches of the run left in
// the group counters (sum of forward_chain_arrivals over them), `launch` the number of those launches.
// The word at forward_chain_status_offset() inside `sync` is a status word: 0, or non-zero when
// a launch gave up (an XCD did not receive exactly 32 of the 256 workgroups, or a wait ran into
// its wall-clock bound); results are then invalid.  Launches that overlap
// on the device would wait for each other's compute units: the caller orders them.
struct ChainStep {
  float* out;
  float* gates;
};
// Bound of every wait inside a resident launch, in ticks of the 100 MHz wall clock (negative: the
// default of 0.5 s).  0 makes every wait give up at once.
void set_resident_wait_ticks(long long ticks);
bool can_run_forward_chain(const Dims& d);
int forward_chain_max_steps();
size_t forward_chain_ring_bytes(const Dims& d);
size_t forward_chain_sync_bytes();
size_t forward_chain_status_offset();
unsigned forward_chain_arrivals(int steps);
hipError_t launch_forward_chain(const Dims& d, const void* Wp, const float* bp, const float* x_first, const float* src_unit,
                                const ChainStep* steps, int count, void* ring, unsigned* sync, unsigned base,
                                unsigned launch, hipStream_t st);

// A run of (forward operation keeping the internal state, backward operation) pairs for steps
// s_hi, s_hi - 1, ..., in one weight-gradient chunk or two consecutive ones, in one launch with both weight
// operands resident on the chip (shapes for which can_run_sweep() holds).  src[j] is the unit
// holding the state before step s_hi - j; the internal states never reach memory; everything a
// backward step writes (dG, its transposed copies, y_out, the running dc) is written as by
// launch_backward.  sync/base/launch as for launch_forward_chain, whose counters it shares: a
// launch of n steps leaves forward_chain_arrivals(n) arrivals.
struct SweepArgs {
  const void* Wp;
  const void* WTh;
  const float* bp;
  const float* x;          // x of step 1
  const float* dy;         // plane of step dy_first first, or NULL
  int dy_first, dy_is_h;
  float* dc;
  float* y_out;            // plane of step 1 first, or NULL
  const void* dG_next;     // dG block of step s_hi + 1, or NULL for the last step of the sequence
  void* dG_chunk[2];       // the two chunk buffers of each operand, indexed by chunk parity: a launch may cross
  void* dGT[2];            // from one chunk of steps into the one below
  void* aT[2];
  unsigned* sync;
  unsigned base, launch;
  int s_hi, count;
  const float* const* src;
  const float* const* state;   // NULL, or per step the unit where an earlier launch stored the internal state:
                               // then no forward operation is run (can_run_backward_sweep() shapes)
};
bool can_run_sweep(const Dims& d);
bool can_run_backward_sweep(const Dims& d);
int sweep_max_steps();
hipError_t launch_sweep(const Dims& d, const SweepArgs& a, hipStream_t st);

// out[slot*B + b][n] = sum_k dG[slot*BP + b][k] * WT[n][k] for slot < nslots, b < B, n < N;
// ld_out = row stride of out.  Used for dx (WT = WTx, N = I) and for dh_0 (WT = WTh, N = H).
// dx of a chunk of steps: launch_dgrad_gemm(WTx, I, ...) on most shapes; where the output has few
// 256 x 256 blocks and K = 4H is long, the blocked GEMM with every block's K shared out, its partial
// blocks in `scratch` (device memory the caller lends until the call's work is done; contents lost).
bool dx_gemm_uses_blocks(const Dims& d, size_t scratch_bytes);
hipError_t launch_dx_gemm(const Dims& d, const void* WTx, const void* dG, int nslots, float* dx, void* scratch,
                          size_t scratch_bytes, hipStream_t st);
hipError_t launch_dgrad_gemm(const Dims& d, const void* WT, int N, const void* dG, int nslots, float* out,
                             int ld_out, hipStream_t st);

// x of `nslots` consecutive steps -> rows [0,NX) of aT, and ones into row NX+HP for the same columns.
hipError_t launch_transpose_x(const Dims& d, const float* x_first, int nslots, void* aT, hipStream_t st);

// Zeroes columns [c0, c1) of every row of the two weight-gradient operands dGT and aT (c1 <= KC).
hipError_t launch_zero_operand_columns(const Dims& d, void* dGT, void* aT, int c0, int c1, hipStream_t st);

// Tile-ordered running sum of [dW | db] (+)= dGT * aT^T over K = nslots*B columns.
// launch_wgrad_finish writes the caller's row-major dW_ih, dW_hh and db from it.
size_t wgrad_accumulator_bytes(const Dims& d);
hipError_t launch_wgrad(const Dims& d, const void* dGT, const void* aT, int nslots, int accumulate, float* dWacc,
                        hipStream_t st);
hipError_t launch_wgrad_finish(const Dims& d, const float* dWacc, float* dW_ih, float* dW_hh, float* db,
                               hipStream_t st);

// One [B,H] plane: dst = src (accumulate 0), dst += src (1), dst = 0 (2; src unused).
hipError_t launch_copy_plane(const Dims& d, const float* src, float* dst, int accumulate, hipStream_t st);

}  // namespace mebptt
