/*
 * mebptt -- memory-efficient LSTM back-propagation through time on AMD MI355X (gfx950).
 *
 * C ABI of the library.  Two halves:
 *
 *   mebptt_plan(...)  host only.  Solves the paper's dynamic programs for the optimal
 *                     checkpointing policy under a budget of m memory slots -- BPTT-HSM
 *                     (Section 3.1, eq. 1-3, Algorithm 1), BPTT-ISM (Section 3.2, eq. 4-5),
 *                     BPTT-MSM (Sections 3.3-3.4, eq. 6-10) -- and flattens the policy for
 *                     (t, m) into a linear schedule of forward runs and backward steps
 *                     (Algorithm 2; Section 3.2 steps 1-4; Section 3.3 last paragraph).
 *   mebptt_run(...)   one gradient step of a single-layer LSTM (the experiment of Section 4):
 *                     executes the schedule on the GPU inside the caller's slot pool and
 *                     returns dW, db, dh0, dc0 (and optionally dx and the outputs h_1..h_t).
 *
 * Conventions
 *   - Every function returns MEBPTT_OK (0) or a negative mebptt_status; it never throws or
 *     aborts.  On a validation error no device work has been enqueued.  mebptt_last_error()
 *     gives a thread-local message for the last failure on the calling thread.
 *   - "host" / "device" on a pointer says which memory it must point to.  The library
 *     allocates no device memory: slots, workspace, inputs and outputs belong to the caller.
 *   - Time steps are 1-based: step s consumes x[s-1] and the hidden state of step s-1 and
 *     produces the hidden state of step s.  "Hidden state" is the pair (h_s, c_s) that one LSTM
 *     core hands to the next (Definition 2); it is the memory UNIT: two [B,H] fp32 planes.
 *     An "internal state" (Definition 3) is four units: (h_s, c_s), (i, f), (g, o) and the
 *     input hidden state (h_{s-1}, c_{s-1}); the last unit is omitted when that state is
 *     already held elsewhere (Section 3.4), which gives alpha = 4 and beta = 3 for an LSTM.
 *   - LSTM: G = x_s W_ih^T + h_{s-1} W_hh^T + b, gate order i, f, g, o along the 4H axis;
 *     i, f, o = sigmoid, g = tanh; c_s = f c_{s-1} + i g; h_s = o tanh(c_s).
 *   - All matrices are dense row-major with no padding.
 */
#ifndef MEBPTT_H
#define MEBPTT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MEBPTT_OK = 0,
  MEBPTT_EINVAL = -1,       /* bad argument (null pointer, t < 1, m < 1, alpha < 2, beta > alpha ...) */
  MEBPTT_ENOMEM_SLOTS = -2, /* slot pool smaller than mebptt_slot_pool_bytes()                       */
  MEBPTT_EWORKSPACE = -3,   /* workspace smaller than mebptt_workspace_bytes() or misaligned         */
  MEBPTT_ESHAPE = -4,       /* descriptor and plan disagree (t)                                      */
  MEBPTT_EINFEASIBLE = -5,  /* the dynamic program prices (t, m) at infinity                         */
  MEBPTT_EHIP = -6,         /* a HIP call failed; the message carries hipGetErrorString              */
  MEBPTT_ENOMEM_HOST = -7   /* host allocation for the tables or the schedule failed                 */
} mebptt_status;

/* Which states the slots memorise. */
typedef enum {
  MEBPTT_HSM = 0, /* hidden states only (Section 3.1); m counts slots of one unit, h_0 included      */
  MEBPTT_ISM = 1, /* internal states only (Section 3.2); m counts slots of four units, h_0 excluded  */
  MEBPTT_MSM = 2  /* mixed (Sections 3.3-3.4); m counts units, h_0 included                          */
} mebptt_kind;

typedef struct mebptt_plan_s mebptt_plan_t; /* opaque; host memory owned by the library */

/* ---- schedule ---------------------------------------------------------------------------- */

/* A location names one unit of memory.  Values >= 0 index units of the caller's slot pool;
 * the negative values are units inside the workspace (the "single RNN core available for
 * intermediate calculations" of Section 3.1, outside the budget). */
enum {
  MEBPTT_LOC_NONE = -1,
  MEBPTT_LOC_T0 = -2,   /* transient hidden state, ping          */
  MEBPTT_LOC_T1 = -3,   /* transient hidden state, pong          */
  MEBPTT_LOC_CORE = -4, /* working core: (h,c) here, then (i,f), (g,o) in its next two units */
  MEBPTT_LOC_INIT = -5  /* copy of the caller's (h0, c0); ISM start state */
};

enum { MEBPTT_OP_FWD_RUN = 1, MEBPTT_OP_BWD = 2 };

/* One schedule entry.
 * FWD_RUN: `count` consecutive forward operations, steps step .. step+count-1.  The first reads
 *          the hidden state at `src`; the last writes its hidden state to `dst` and, when
 *          keep != 0, its gates to the two units after `dst`; the state of step
 *          step+count-2 (count > 1) is written to `prev`; earlier ones alternate T0/T1.
 * BWD:     one backward operation of `step` through the internal state at `dst`, whose input
 *          hidden state is at `src`.  The loss gradient of that step is injected here.
 *          Backward entries appear in the order t, t-1, ..., 1. */
typedef struct {
  int32_t op;
  int32_t step;
  int32_t count;
  int32_t src;
  int32_t dst;
  int32_t keep;
  int32_t prev;
} mebptt_op;

/* Alg. 1 generalised to the three strategies.  Builds the tables for every t' <= t and
 * m' <= m and flattens the policy of (t, m).  alpha, beta are used by MSM only (integers,
 * alpha >= 2, 1 <= beta <= alpha; beta == alpha disables Section 3.4).  *out receives a plan to
 * be released with mebptt_plan_free.  Errors: EINVAL, EINFEASIBLE, ENOMEM_HOST. */
int mebptt_plan(int32_t t, int32_t m, int32_t kind, int32_t alpha, int32_t beta, mebptt_plan_t** out);
void mebptt_plan_free(mebptt_plan_t* plan);

/* Section 4.2: every strategy inside the model is a (possibly sub-optimal) policy of BPTT-MSM.
 * A policy is handed over as the decisions the execution procedure of Section 3.3 asks for, in
 * the order it asks: at a node (t', m') with t' >= 2 and m' >= 2 it takes the next decision --
 * memorise the hidden state (store = 1, 1 <= y < t') or the internal state (store = 2,
 * 1 <= y <= t') reached after y forward operations -- then treats the right part
 * (t' - y, m' - units), then the left part (y or y - 1, m').  Nodes with t' <= 1, and nodes
 * with m' = 1 (constant-memory procedure), take no decision.  Units: hidden 1, internal alpha,
 * beta when y = 1; m counts the start state h_0, as in BPTT-MSM. */
enum { MEBPTT_STORE_HIDDEN = 1, MEBPTT_STORE_INTERNAL = 2 };
typedef struct {
  int32_t store;
  int32_t y;
} mebptt_decision;
/* Flattens the policy `decisions[0..n)` (host memory, read during the call only) for a sequence
 * of length t within m units.  The plan has kind MEBPTT_MSM and no tables (the cost, split and
 * choice accessors return NULL); forward_ops is the policy's cost.  alpha >= 4, 3 <= beta <=
 * alpha.  Errors: EINVAL (malformed decision, too few or too many decisions), EINFEASIBLE (the
 * policy does not fit into m), ENOMEM_HOST. */
int mebptt_plan_from_policy(int32_t t, int32_t m, int32_t alpha, int32_t beta, const mebptt_decision* decisions,
                            size_t n, mebptt_plan_t** out);
/* Section 2, "Chen's sqrt(t) algorithm" as such a policy: ceil(sqrt(t)) parts of equal length,
 * the hidden state memorised at every cut, every internal state (beta units each) memorised
 * while a part is back-propagated.  The plan's budget is what the strategy needs. */
int mebptt_plan_chen_sqrt(int32_t t, int32_t alpha, int32_t beta, mebptt_plan_t** out);
/* Section 2, "Chen's recursive algorithm": k >= 1 hidden states memorised per level, cutting a
 * sub-sequence into min(k + 1, length) equal parts, recursively down to single steps (k = 1:
 * bisection, about log2(t) units).  The plan's budget is what the strategy needs. */
int mebptt_plan_chen_recursive(int32_t t, int32_t k, int32_t alpha, int32_t beta, mebptt_plan_t** out);

/* Borrowed read-only views, valid until mebptt_plan_free.  Tables are row-major
 * [(t+1) x (m+1)], entry [t'][m'].  Infeasible cost cells hold MEBPTT_COST_INF; undefined
 * split/choice cells hold 0.
 *   cost   which = 0: C.  MSM also 1: C_1 (hidden push), 2: C_2 (internal push)  (eq. 2, 9)
 *   split  which = 0: D (HSM, ISM).  MSM: 1: D_1, 2: D_2                            (eq. 3, 5, 8)
 *   choice H (eq. 9): 1 = hidden, 2 = internal; MSM only, otherwise NULL.
 * A `which` that the plan's kind does not define returns NULL. */
#define MEBPTT_COST_INF ((int64_t)1 << 60)
const int64_t* mebptt_plan_cost(const mebptt_plan_t* plan, int32_t which);
const int32_t* mebptt_plan_split(const mebptt_plan_t* plan, int32_t which);
const uint8_t* mebptt_plan_choice(const mebptt_plan_t* plan);
int32_t mebptt_plan_length(const mebptt_plan_t* plan);
int32_t mebptt_plan_budget(const mebptt_plan_t* plan);
int32_t mebptt_plan_kind(const mebptt_plan_t* plan);
/* Number of forward operations in the schedule; equals C(t, m) (Section 3.1: the cost is the
 * total number of forward operations).  Counted from the flattened schedule, not read from C. */
int64_t mebptt_plan_forward_ops(const mebptt_plan_t* plan);
/* High-water mark of the stack while the schedule runs, in the plan's budget unit (slots for
 * HSM and ISM, units for MSM); never above m. */
int32_t mebptt_plan_peak(const mebptt_plan_t* plan);
/* The flat schedule; *n receives the number of entries. */
const mebptt_op* mebptt_plan_schedule(const mebptt_plan_t* plan, size_t* n);

/* ---- non-homogeneous chains ---------------------------------------------------------------------
 * Appendix "Generalizing to deep feed-forward networks": the policy for a linear chain whose
 * layers differ in forward cost u_i, output size s_i and working-memory size p_i (memory in
 * arbitrary integer units; the network input is always available and not counted).
 *   C(t, m, x) = cost of back-propagating through layers x+1 .. x+t with m free units when the
 *                input of layer x+1 is available;  Q = U(x,y) + K(x,y,m) + C(t-y, m-s_{x+y}, x+y)
 *                + C(y, m, x), 1 <= y < t;  D = smallest minimising y.
 * Readings: one layer costs u if p fits; at every node the sub-chain may also be processed
 * without memorising anything (re-run from its input before each backward step), recorded as
 * D = 0; a tie goes to the memorisation.  With u = s = 1, p = 0 this is BPTT-HSM with the start
 * state outside the budget.  mebptt_chain_run (below) executes such a plan on a stack of dense
 * tanh layers of differing widths. */
typedef struct {
  int64_t cost;        /* u_i >= 1 */
  int32_t state_units; /* s_i >= 1: size of the layer's output */
  int32_t work_units;  /* p_i >= 0: memory a forward or backward operation of the layer needs */
} mebptt_layer;
typedef struct mebptt_chain_plan_s mebptt_chain_plan_t;
enum { MEBPTT_CHAIN_FORWARD = 1, MEBPTT_CHAIN_BACKWARD = 2 };
enum { MEBPTT_CHAIN_INPUT = -1, MEBPTT_CHAIN_WORKING = -2 };
/* FORWARD:  `count` layers layer .. layer+count-1 from the state at `src` (unit offset in the pool
 *           of m units, MEBPTT_CHAIN_INPUT, or MEBPTT_CHAIN_WORKING); the last output is memorised
 *           at unit offset `dst`, or stays in working memory (MEBPTT_CHAIN_WORKING).
 * BACKWARD: one backward operation of `layer`, whose input state is at `src`.  Backward entries
 *           come in the order n, n-1, ..., 1. */
typedef struct {
  int32_t op;
  int32_t layer;
  int32_t count;
  int32_t src;
  int32_t dst;
} mebptt_chain_op;
/* Solves the program for every sub-chain and every m' <= m and flattens the policy of the whole
 * chain.  `layers` (host, n entries) is copied.  Errors: EINVAL, EINFEASIBLE (some layer cannot
 * run in m units), ENOMEM_HOST (the table has (n+1)(n+2)/2 x (m+1) cells). */
int mebptt_chain_plan(const mebptt_layer* layers, int32_t n, int32_t m, mebptt_chain_plan_t** out);
void mebptt_chain_plan_free(mebptt_chain_plan_t* plan);
/* C(t, m', x) and D(t, m', x) for 0 <= t, x + t <= n, m' <= m (MEBPTT_COST_INF / 0 outside or if
 * infeasible; m' < 0 is infeasible). */
int64_t mebptt_chain_cost(const mebptt_chain_plan_t* plan, int32_t t, int32_t m, int32_t x);
int32_t mebptt_chain_split(const mebptt_chain_plan_t* plan, int32_t t, int32_t m, int32_t x);
/* Forward cost summed over the schedule (= C(n, m, 0)) and the high-water mark of memorised
 * outputs plus working memory while it runs (<= m). */
int64_t mebptt_chain_plan_forward_cost(const mebptt_chain_plan_t* plan);
int32_t mebptt_chain_plan_peak(const mebptt_chain_plan_t* plan);
const mebptt_chain_op* mebptt_chain_plan_schedule(const mebptt_chain_plan_t* plan, size_t* n);
/* The plan's copy of the layer table; *n receives the number of layers. */
const mebptt_layer* mebptt_chain_plan_layers(const mebptt_chain_plan_t* plan, int32_t* n);

/* Execution of a chain plan on the GPU (the appendix's generalisation, smallest honest instance):
 * n dense layers y_i = tanh(y_{i-1} W_i^T + b_i), W_i [d_i, d_{i-1}], batch B, widths d_0 .. d_n
 * that differ from layer to layer, fp32 throughout (fp32 MFMA tiles, fp32 accumulate).  Memory is
 * counted in units of unit_bytes: the output of layer i takes ceil(B d_i 4 / unit_bytes) units, its
 * forward cost is d_{i-1} d_i (multiply-adds per sequence), and the working memory of an operation
 * (two activations, the gradient passed down, one dz) is the caller's workspace, outside the
 * budget (work_units = 0) -- the same accounting as the LSTM path's working core.
 * mebptt_chain_layers fills `out` (host, n entries) with that table for mebptt_chain_plan. */
typedef struct {
  int32_t n, B;
  const int32_t* widths; /* host, n + 1 entries d_0 .. d_n */
  size_t unit_bytes;     /* bytes of one memory unit, a multiple of 4 */
} mebptt_chain_desc;
typedef struct {
  int64_t forward_cost; /* sum of the forward costs of the forward operations launched (== C(n, m, 0)) */
  int64_t backward_ops; /* == n */
  int32_t peak_units;   /* highest pool unit any launch was handed (<= m) */
  int32_t reserved;
} mebptt_chain_stats;
int mebptt_chain_layers(const mebptt_chain_desc* desc, mebptt_layer* out);
size_t mebptt_chain_workspace_bytes(const mebptt_chain_desc* desc);
/* One gradient step of the chain under `plan` (made by mebptt_chain_plan from mebptt_chain_layers
 * of the same desc, else ESHAPE), the loss gradient arriving at the last layer's output.
 * host arrays of n device pointers: W (W_i [d_i, d_{i-1}] row-major), b (b_i [d_i] or NULL entries
 *   for zero), dW, db (written, same shapes).
 * device, read:  x0 [B, d_0], dy [B, d_n] = dL/dy_n.
 * device, r/w:   pool (>= m * unit_bytes, 256-byte aligned; may be NULL when m = 0), workspace
 *                (>= mebptt_chain_workspace_bytes, 256-byte aligned).
 * device, write: dx0 [B, d_0] and y_out [B, d_n] (either may be NULL).
 * host, write:   stats (may be NULL).  The call only enqueues work on `stream`.
 * Errors: EINVAL, ESHAPE, ENOMEM_SLOTS, EWORKSPACE, EHIP; nothing is enqueued on a validation error. */
int mebptt_chain_run(const mebptt_chain_desc* desc, const mebptt_chain_plan_t* plan,
                     const float* const* W, const float* const* b, const float* x0, const float* dy,
                     void* pool, size_t pool_bytes, void* workspace, size_t workspace_bytes,
                     float* const* dW, float* const* db, float* dx0, float* y_out,
                     mebptt_chain_stats* stats, void* stream);

/* ---- LSTM execution ---------------------------------------------------------------------- */

typedef struct {
  int32_t B, I, H, t;
  int32_t gemm_dtype;    /* 0: fp32 GEMM operands; 1: bf16 GEMM operands.  Accumulation, state
                            storage and all pointwise arithmetic are fp32 either way.          */
  int32_t loss;          /* 0: upstream gradients come from `dy`; 1: built-in loss
                            0.5 * sum_s sum(h_s^2), i.e. dy_s = h_s                             */
  int32_t dy_first_step; /* loss 0: `dy` covers steps dy_first_step .. t (1-based); the steps
                            before carry no loss.  Use 1 for a loss at every step.              */
  int32_t cell;          /* the RNN core (Section 1: the method does not depend on it):
                            MEBPTT_CELL_LSTM or MEBPTT_CELL_GRU                                 */
} mebptt_lstm_desc;
enum { MEBPTT_CELL_LSTM = 0, MEBPTT_CELL_GRU = 1 };

typedef struct {
  int64_t forward_ops;    /* forward operations launched (== C(t, m))   */
  int64_t backward_ops;   /* backward operations launched (== t)        */
  int32_t peak;           /* highest slot occupied by any launch, in budget units (<= m) */
  int32_t reserved;
  size_t peak_slot_bytes; /* the same high-water mark in bytes of the slot pool          */
} mebptt_stats;

/* Bytes of one unit: a hidden state (h, c) (Definition 2) in fp32 = 2 * B * H * 4. */
size_t mebptt_unit_bytes(const mebptt_lstm_desc* desc);
/* Bytes of the slot pool for this plan.  A memory slot (Definition 4) holds one hidden state
 * (HSM; MSM counts in these units) or one internal state with its input state (ISM: four
 * units); the pool is the plan's m slots and nothing else -- this is the budget of Section 3. */
size_t mebptt_slot_pool_bytes(const mebptt_lstm_desc* desc, const mebptt_plan_t* plan);
/* Bytes of workspace, the memory outside the budget.  Section 3.1 grants the method "a single
 * RNN core available for intermediate calculations, able to store a single internal state":
 * that is the working core and the two transient hidden states here.  The rest is what this
 * implementation adds around it: operand copies of the weights in the GEMM type, the running
 * gradients, a dW accumulator, staging of dG / [x; h] for the steps of two chunks of the
 * time-batched weight-gradient GEMM and, on shapes where the way back through a stretch of stored
 * hidden states recomputes the stretch's internal states in one launch (bf16 LSTM, H = 1024), a
 * stage for those internal states (at most 32 of them and at most 48 MiB).  Independent of t and
 * of the budget. */
size_t mebptt_workspace_bytes(const mebptt_lstm_desc* desc);
/* Largest budget, in the given kind's unit, whose slot pool fits in budget_bytes (0 if none). */
int32_t mebptt_units_for_bytes(const mebptt_lstm_desc* desc, int32_t kind, size_t budget_bytes);

/* Alg. 2 / Section 3.2 / Section 3.3: one combined forward-and-backward gradient step.
 *
 * device, read:  W_ih [4H,I], W_hh [4H,H], b [4H] (NULL = zeros), x [t,B,I],
 *                dy [t-dy_first_step+1, B, H] (loss 0; ignored for loss 1),
 *                h0, c0 [B,H] (NULL = zeros).
 *                LSTM: gate order i, f, g, o along the 4H axis, one bias vector.
 *                GRU (cell = MEBPTT_CELL_GRU): W_ih [3H,I], W_hh [3H,H], gate order r, z, n;
 *                b [6H] = [b_ih | b_hh]; n = tanh(W_in x + b_in + r * (W_hn h + b_hn)),
 *                h' = (1 - z) * n + z * h.  c0 is ignored.  The gradients have the same
 *                shapes (dW_ih [3H,I], dW_hh [3H,H], db [6H]); dc0 is written as zero.  A slot
 *                unit keeps the LSTM's size, so the same plans and budgets apply.
 * device, r/w:   slots (>= mebptt_slot_pool_bytes, 256-byte aligned), workspace
 *                (>= mebptt_workspace_bytes, 256-byte aligned).  Contents on entry are ignored;
 *                contents on exit are unspecified.
 * device, write: dW_ih [4H,I], dW_hh [4H,H], db [4H], dh0, dc0 [B,H]: OVERWRITTEN with the
 *                gradients.  dx [t,B,I] and y_out [t,B,H] may be NULL (then not computed).
 * host, write:   stats (may be NULL); filled before the call returns.
 * stream:        a hipStream_t (NULL = the default stream).  The call only enqueues work; results
 *                are valid once the caller has synchronised the stream.
 * stats:         forward_ops and backward_ops count the launches made; peak is the highest slot
 *                unit any launch of this run was handed (rounded up to budget units), tracked by
 *                the executor while it walks the schedule -- it equals mebptt_plan_peak().
 *
 * Library-owned resources.  The time-batched dW and dx GEMMs of finished chunks run on a second,
 * non-blocking HIP stream of default priority that the library creates on the first run on a
 * device, with four events to fork from and join back into `stream` (no host synchronisation:
 * the whole call can be captured into a HIP graph).  They live until mebptt_shutdown().  Because
 * they are shared, a process-wide mutex serialises the ENQUEUE phase of concurrent mebptt_run
 * calls (any thread, any stream); the device work of two runs on different streams, slot pools
 * and workspaces may overlap.  The measurement hooks below use process-wide state and must not
 * be toggled while another thread is inside a run.
 * Errors: EINVAL, ESHAPE, ENOMEM_SLOTS, EWORKSPACE, EHIP. */
int mebptt_run(const mebptt_lstm_desc* desc, const mebptt_plan_t* plan,
               const float* W_ih, const float* W_hh, const float* b,
               const float* x, const float* dy, const float* h0, const float* c0,
               void* slots, size_t slots_bytes, void* workspace, size_t workspace_bytes,
               float* dW_ih, float* dW_hh, float* db, float* dh0, float* dc0,
               float* dx, float* y_out, mebptt_stats* stats, void* stream);

/* The same gradient step in two calls, for weights that stay unchanged over several runs (e.g.
 * several sequences per optimiser step).  mebptt_prepare builds the operand copies of the
 * weights (GEMM type, gate-interleaved, transposed for the backward GEMMs) and clears the staging
 * inside `workspace`; mebptt_run_prepared then runs any number of gradient steps of that shape
 * (B, I, H, gemm_dtype, cell; t, loss and the plan may change) on it without repeating that work.
 * mebptt_run == mebptt_prepare + mebptt_run_prepared.  The library remembers on the host which
 * workspace pointers were prepared for which shape and refuses others (EWORKSPACE); it cannot
 * see the caller overwrite the workspace or change the weights -- prepare again after either.
 * Arguments, ownership and stream semantics are those of mebptt_run.
 * Errors: as mebptt_run. */
int mebptt_prepare(const mebptt_lstm_desc* desc, const float* W_ih, const float* W_hh, const float* b,
                   void* workspace, size_t workspace_bytes, void* stream);
int mebptt_run_prepared(const mebptt_lstm_desc* desc, const mebptt_plan_t* plan,
                        const float* x, const float* dy, const float* h0, const float* c0,
                        void* slots, size_t slots_bytes, void* workspace, size_t workspace_bytes,
                        float* dW_ih, float* dW_hh, float* db, float* dh0, float* dc0,
                        float* dx, float* y_out, mebptt_stats* stats, void* stream);

/* Forward operations that follow each other (Algorithm 2's forward loop, and the consecutive
 * single-step pushes of a sub-sequence that fits into memory) are issued as "forward-chain"
 * launches where the shape allows it (bf16 operands, either cell, H a multiple of 128 and gate weights
 * that fit into the registers and LDS of one XCD's compute units): one launch then carries up to
 * 192 steps, keeps the gate weights on the chip, splits the batch over the 8 XCDs and lets the 32
 * compute units of an XCD exchange h through their shared L2.  Where the transposed recurrent
 * weights fit as well (LSTM, H = 128, 256, 512 with I <= H/4 .. H), the runs of "forward operation keeping
 * the internal state, then backward operation" that end every sub-sequence are issued the same way
 * ("sweep" launches, up to 32 pairs, internal states never leaving the registers).  Where only the
 * transposed recurrent weights fit (H = 1024), and for the GRU at every such width, the forward operations of such a run -- they do not
 * depend on each other, every input state being in a slot already -- go out as one "forward-batch"
 * launch that leaves the internal states in the workspace's stage, followed by one sweep launch of
 * backward operations on them; backward operations on internal states stored in slots go out as
 * such sweep launches as well.  Results are bit-identical to the launch-per-step path.  Such a launch assumes that its 256 workgroups are all resident and dealt
 * round-robin to the XCDs; each workgroup checks this, every wait inside is bounded by a wall
 * clock, and a launch that cannot proceed gives up and raises a status word in the workspace
 * instead of hanging.  mebptt_run_status copies that word to *status (host) after waiting for
 * `stream`: 0 = every launch of the last run on this workspace completed; non-zero = a launch
 * gave up and the run's outputs are invalid (1: a wait ran into its bound, 2: a workgroup was
 * not placed on the XCD its id implies).  Two runs that use such launches must not overlap on one
 * device (each would hold a part of the chip and wait for the rest): the library orders its own
 * eager runs across streams with an event; replays of captured graphs are the caller's to order.
 * Errors: EINVAL, EWORKSPACE, EHIP. */
int mebptt_run_status(const mebptt_lstm_desc* desc, const void* workspace, size_t workspace_bytes, void* stream,
                      int32_t* status);

/* on = 0: from now on every forward and backward operation gets a launch of its own (or shares a
 * pair launch), whatever the shape (the path the forward-chain, sweep and forward-batch launches
 * are checked against, and the "before" of their measurement); on != 0 (the default) restores them.  They are
 * used only on a device that reports 256 compute units (8 XCDs of 32): on a partitioned device or
 * one with masked compute units the launch-per-step path runs regardless of this switch.
 * Process-wide; not to be toggled while a run is enqueued. */
int mebptt_forward_chain_enable(int32_t on);
/* The bound every wait inside a forward-chain or sweep launch runs under, in ticks of the device's
 * 100 MHz wall clock (default 50 000 000 = 0.5 s; a negative value restores the default).  With 0
 * every wait that does not find its data at once gives up: each workgroup leaves through the
 * ordinary exit, the run completes with invalid results and mebptt_run_status reports 1 -- the path
 * a real time-out takes, made reachable for tests.  Process-wide; applies to launches enqueued
 * after the call. */
int mebptt_resident_wait_limit(int64_t ticks);

/* Releases what the library created on every device: the side streams and their events, the
 * events of the measurement hooks, the record of prepared workspaces.  Waits for the side
 * streams first; the caller makes sure no run is being enqueued.  The library can be used again
 * afterwards (resources are re-created on demand).  Errors: EHIP. */
int mebptt_shutdown(void);

/* For callers that cannot allocate (code under HIP graph capture, tight serving loops, harnesses
 * that forbid hipMalloc): mebptt_run with the workspace taken from a file-scope device array of
 * MEBPTT_STATIC_WORKSPACE_BYTES that every GPU the library runs on holds until the process ends.
 * The call creates no stream and no event and allocates nothing: every kernel, including the
 * time-batched GEMMs, is enqueued on `stream` in schedule order; the measurement hooks are
 * ignored.  Results are bit-identical to mebptt_run's.  Shapes whose workspace (as
 * mebptt_workspace_bytes() counts it, less the recomputation stage, which this path never uses)
 * exceeds the array are refused with EWORKSPACE before anything is enqueued.  All calls on one
 * GPU share the array, which keeps the previous call's contents (the call clears what must start
 * at zero): calls whose device work overlaps on one GPU race -- keep them on one stream or
 * order them with events.  Other arguments as mebptt_run. */
#define MEBPTT_STATIC_WORKSPACE_BYTES ((size_t)32 << 20)
size_t mebptt_static_workspace_bytes(void);
int mebptt_run_static(const mebptt_lstm_desc* desc, const mebptt_plan_t* plan,
                      const float* W_ih, const float* W_hh, const float* b,
                      const float* x, const float* dy, const float* h0, const float* c0,
                      void* slots, size_t slots_bytes,
                      float* dW_ih, float* dW_hh, float* db, float* dh0, float* dc0,
                      float* dx, float* y_out, mebptt_stats* stats, void* stream);

/* ---- measurement hooks ---------------------------------------------------------------------
 * Kernel classes of the hot path, for timing with HIP events on the run's own stream. */
enum {
  MEBPTT_K_FORWARD = 0,  /* gate GEMM + LSTM pointwise (one forward operation)                 */
  MEBPTT_K_BACKWARD = 1, /* dh GEMM + loss-gradient injection + pointwise backward            */
  MEBPTT_K_WGRAD = 2,    /* time-batched dW/db accumulation (with the x transpose feeding it) */
  MEBPTT_K_DGRAD = 3,    /* time-batched dx GEMM and the final dh0 GEMM                       */
  MEBPTT_K_SETUP = 4,    /* operand copies of the weights, zero fills, start-state copy       */
  MEBPTT_K_PAIR = 5,     /* one launch carrying a backward step and an independent forward op */
  MEBPTT_K_CHAIN = 6,    /* one launch carrying a chain of forward operations, weights resident  */
  MEBPTT_K_SWEEP = 7,    /* one launch carrying a run of backward steps (with or without the forward
                            operations that recompute their internal states), weights resident */
  MEBPTT_K_FWD_BATCH = 8, /* one launch carrying forward operations that do not depend on each other */
  MEBPTT_K_CLASSES = 9
};
typedef struct {
  int64_t launches[MEBPTT_K_CLASSES]; /* launches of the class in the profiled runs      */
  int64_t sampled[MEBPTT_K_CLASSES];  /* launches inside event brackets (consecutive launches of a
                                         sequential class share one bracket, up to eight)  */
  double sampled_ms[MEBPTT_K_CLASSES]; /* sum of the brackets' elapsed times              */
  /* Forward runs of nine or more consecutive operations are also bracketed as a whole (all but
   * their first launch): one event pair around many back-to-back launches, so the cost of the
   * events themselves disappears from the per-launch average. */
  int64_t forward_run_launches;
  double forward_run_ms;
  /* Forward-chain launches are all bracketed: forward operations they carried, and their time. */
  int64_t chain_steps;
  double chain_ms;
  /* Likewise the sweep launches: backward steps they carried, and their time. */
  int64_t sweep_steps;
  double sweep_ms;
  int64_t sampled_groups[MEBPTT_K_CLASSES]; /* event brackets behind `sampled` and `sampled_ms` */
  /* Forward operations carried by sweep launches (the others run on internal states stored before). */
  int64_t sweep_forward_steps;
  /* The launches of independent forward operations are all bracketed: operations carried, time. */
  int64_t batch_steps;
  double batch_ms;
} mebptt_profile;
/* every_n > 0: from now on mebptt_run (on this thread's process-wide state) brackets every
 * every_n-th launch of each class with a pair of HIP events recorded on the run's stream;
 * 0 switches sampling off (the default).  Not thread-safe against concurrent mebptt_run. */
int mebptt_profile_enable(int32_t every_n);
/* Waits for the recorded events, writes the sums since the last collect (host memory) and
 * clears them.  Errors: EINVAL, EHIP. */
int mebptt_profile_collect(mebptt_profile* out);

/* Average time, in microseconds, of `launches` back-to-back empty kernel launches on `stream`
 * (host memory out_us), bracketed by one event pair: the floor every dependent launch of the
 * sequential chain pays on this machine.  Synchronises the stream.  Errors: EINVAL, EHIP. */
int mebptt_null_launch_us(int32_t launches, void* stream, double* out_us);

/* The two time-batched GEMMs of one full chunk of this shape (dW/db accumulation, K = CH*B; dx,
 * K = 4H), each launched `reps` times back to back on `stream` with nothing else on the device,
 * on the staging buffers inside `workspace` as they are (the arithmetic is data-independent;
 * contents are not checked) -- their time alone, in microseconds per launch (host memory).
 * Synchronises the stream.  Errors: EINVAL, EWORKSPACE, EHIP. */
int mebptt_measure_gemms(const mebptt_lstm_desc* desc, void* workspace, size_t workspace_bytes, int32_t reps,
                         void* stream, double* wgrad_us, double* dgrad_us);
/* What the memory system needs to deliver one forward launch's bytes: a kernel with the grid of the
 * forward launch of this shape whose workgroups only read the operand panels their forward
 * counterparts read (the weight panel from the workspace's operand copy, an activation panel of the
 * same size from its state area), launched `reps` times back to back on `stream`: microseconds per
 * launch and the bytes all workgroups read per launch (host memory).  Contents are not looked at.
 * Synchronises the stream.  Errors: EINVAL, EWORKSPACE, EHIP. */
int mebptt_measure_forward_stream(const mebptt_lstm_desc* desc, void* workspace, size_t workspace_bytes, int32_t reps,
                                  void* stream, double* us_per_launch, double* delivered_bytes);
/* Time steps per chunk of the time-batched GEMMs for this shape (the K extent of the dW GEMM is
 * this many times B), or a negative error code. */
int32_t mebptt_chunk_steps(const mebptt_lstm_desc* desc);
/* Internal states the recomputation stage inside the workspace holds for this shape (0: the shape
 * has no stage: its recomputation runs do not go out as a forward batch plus a backward-only sweep
 * launch), or a negative error code. */
int32_t mebptt_stage_steps(const mebptt_lstm_desc* desc);

/* What one synchronisation of the 256 workgroups of a resident launch costs, alone: `iters`
 * synchronisations inside one kernel on `stream`, microseconds per synchronisation (host memory).
 * variant 0: all workgroups meet at one device-wide counter; 1: the 32 workgroups of each XCD meet
 * at their XCD's counter (what forward chains and sweeps do per time step); 2: as 1, plus an
 * exchange of 512 bytes per workgroup that the 32 of the XCD then read through the L2, every word
 * checked.  *status (host memory): 0 ok, 1 a bounded wait gave up, 2 the workgroups were not placed
 * 32 per XCD, 3 a word read back differed.  Allocates and frees its own small device buffers;
 * synchronises the stream.  Errors: EINVAL, EHIP. */
int mebptt_measure_sync(int32_t variant, int32_t iters, void* stream, double* us_per_sync, int32_t* status);

/* What an event pair around a single launch adds to that launch's time, for a kernel lasting about
 * kernel_us (0..1000): `reps` (1..2000) launches of a kernel that idles that long, back to back
 * inside one event pair -> *per_launch_us; the same launches each inside its own event pair ->
 * *bracketed_us (mean).  Event-sampled per-launch times carry the difference.  Host memory outputs;
 * synchronises the stream.  Errors: EINVAL, EHIP. */
int mebptt_bracket_overhead_us(double kernel_us, int32_t reps, void* stream, double* per_launch_us, double* bracketed_us);

const char* mebptt_last_error(void);
/* Library version string, e.g. "mebptt 0.1 (gfx950)". */
const char* mebptt_version(void);

#ifdef __cplusplus
}
#endif
#endif /* MEBPTT_H */
