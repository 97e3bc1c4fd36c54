/*
 * lopt.h -- C boundary of the learned-optimizer step library for AMD MI355X (gfx950).
 *
 * One call, lopt_step(), performs the whole per-parameter optimizer step of the
 * paper's two learned optimizers, small_fc_lopt and VeLO, for a list of parameter
 * tensors: accumulator update, feature statistics, feature normalization, the
 * per-element MLP and the exponentiated parameter update (paper: section "CUDA
 * Implementation", figure "Overview of the Learned Optimizer (LO) update
 * mechanism", appendix "Features for learned optimizer input").
 *
 * General conventions
 *  - Every pointer named *_host is host memory; params, grads, state blobs and the
 *    workspace are DEVICE memory owned by the caller (fp32, 16-byte aligned).
 *  - The library owns only the lopt_ctx: a device copy of the optimizer's weights,
 *    a cached device table describing the tensor list, a pinned staging buffer and
 *    one extra stream with its events (plus one fixed scratch array per GPU, see lopt_step_static).
 *    lopt_step allocates device memory only when the tensor list changes.
 *  - All device work is ordered by the HIP stream passed in (a hipStream_t cast to
 *    void*, NULL = default stream): it starts after everything enqueued on that
 *    stream before the call and is complete before anything enqueued on it after
 *    the call. For large small_fc_lopt lists lopt_step cuts the list into groups and
 *    runs the HBM-bound passes of one group on a library-owned second stream beside
 *    the compute-bound apply pass of the previous group; that stream forks from and
 *    joins back into the caller's stream through events inside the same call.
 *    No call synchronizes the host with the device except when a cached table has to
 *    be rewritten while its previous upload is still in flight.
 *  - Every call validates its arguments on the host before launching anything and
 *    returns a status; nothing throws or aborts across this boundary, and
 *    lopt_last_error() gives a message. After a status that comes from that validation
 *    (LOPT_EINVAL, LOPT_ESHAPE, LOPT_ESTATE, LOPT_ELIMIT, and LOPT_ENOMEM / LOPT_EHIP raised
 *    while tables are prepared) params and state are untouched. A HIP error raised later,
 *    while a step's kernels are being enqueued, leaves params and state partly updated:
 *    the library joins its second stream back into the caller's, marks the context failed,
 *    and every later step through it returns LOPT_EHIP.
 *  - A context is not thread-safe: calls on one context must not overlap on the host, and
 *    steps enqueued through one context on different streams are not ordered with respect to
 *    each other by the library (they share the context's tables and the caller's workspace).
 *    Use one context per concurrently running optimizer.
 *  - Results are deterministic: the same inputs give bit-identical outputs (all
 *    reductions have a fixed order; no floating-point atomics).
 *  - A tensor is described as a row-major rows x cols matrix. The caller flattens:
 *    1-D [n] -> 1 x n; ndim > 2 -> (dim0, product of the rest); leading size-1 dims
 *    squeezed. `ndim` is the squeezed rank (used only by VeLO's hypernetwork input).
 *  - rows * cols must be in [1, 2^31 - 1]. A list of zero tensors is a valid no-op.
 */
#ifndef LOPT_H
#define LOPT_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef struct lopt_ctx lopt_ctx; /* opaque, library-owned */

typedef enum {
  LOPT_OK = 0,
  LOPT_EINVAL = 1, /* null pointer, bad struct size, bad scalar, misaligned pointer */
  LOPT_ESHAPE = 2, /* rows/cols out of range */
  LOPT_ESTATE = 3, /* weights blob of the wrong size for this configuration */
  LOPT_ENOMEM = 4, /* host or device allocation failed */
  LOPT_EHIP = 5,   /* a HIP runtime call failed (message has the HIP error string) */
  LOPT_ELIMIT = 6  /* lopt_step_static: the tensor list needs more scratch than the fixed array holds */
} lopt_status;

typedef enum { LOPT_SMALL_FC = 0, LOPT_VELO = 1 } lopt_kind;

/* Apply kernel for small_fc_lopt with hidden width 32 (other widths and VeLO have one kernel each; VeLO honours
 * LOPT_APPLY_VALU). None changes what is computed beyond rounding. */
typedef enum {
  LOPT_APPLY_AUTO = 0,      /* = LOPT_APPLY_MFMA_F16S */
  LOPT_APPLY_VALU = 1,      /* fp32 vector ALU */
  LOPT_APPLY_MFMA_F32 = 2,  /* fp32 matrix cores */
  LOPT_APPLY_MFMA_F16S = 3  /* matrix cores on fp16 hi+lo operand pairs, fp32 accumulate; column strips, software-pipelined */
} lopt_apply_kernel;

/* Which pass writes the new momentum / second-moment accumulators M_1..3, V when the apply kernel is one of the two
 * default ones: LOPT_APPLY_MFMA_F16S (small_fc_lopt, hidden 32) or the width-4 VeLO kernel. Every other kernel
 * combination writes them in the statistics pass. The values are the same bit for bit either way: both passes form
 * them with the same fp32 operations from the same inputs. */
typedef enum {
  LOPT_STATE_AUTO = 0,      /* = LOPT_STATE_IN_APPLY */
  LOPT_STATE_IN_STATS = 1,  /* statistics pass reads and writes them (40 bytes per element), apply pass reads them (28) */
  LOPT_STATE_IN_APPLY = 2   /* statistics pass only reads them (24 bytes per element, and a read-only stream reaches a
                               higher share of the HBM rate than a read-write one); the apply pass forms them again and
                               writes them (44 bytes per element) */
} lopt_state_pass;

/* Number of time features tanh(t/x), x in {1,3,10,30,100,300,1e3,3e3,1e4,3e4,1e5}
 * (feature table of small_fc_lopt, row "Time Features"). */
#define LOPT_N_TIME 11
/* Per-element features shared by both optimizers (feature tables: 10 accumulators +
 * 16 accumulator features + parameter + gradient). */
#define LOPT_N_ELEM_FEATS 28
/* MLP input width: 28 + 11 time features = 39 (small_fc_lopt, table row "Total"),
 * 28 + clipped gradient = 29 (VeLO, table row "Total"). */
#define LOPT_D_SMALL_FC 39
#define LOPT_D_VELO 29
/* Loss features of VeLO's hypernetwork: tanh(psi/x), psi = sign(loss) ln(1 + |loss|), x in {1, 3, 10}
 * (the paper's artifact appendix, "Basic Usage": the current loss value is passed to VeLO's step). */
#define LOPT_N_LOSS 3
/* Width of the VeLO hypernetwork's LSTM input: 29 log-statistics + 11 time features
 * + one-hot of min(ndim, 4) + 3 loss features. */
#define LOPT_VELO_LSTM_IN 48

typedef struct {
  uint32_t struct_size; /* = sizeof(lopt_config) */
  uint32_t kind;        /* lopt_kind */
  uint32_t hidden;      /* MLP hidden width H, 1..32 (paper uses 32 for small_fc_lopt) */
  float mom_decay[3];   /* beta_1..3: momentum accumulators (feature tables, "Accumulators") */
  float rms_decay;      /* beta_4: second-moment accumulator */
  float fac_decay[3];   /* beta_5..7: Adafactor row/column accumulators */
  float eps_acc;        /* added inside every reciprocal square root of an accumulator */
  float eps_norm;       /* added inside the normalization square root ("Feature normalization") */
  float exp_mult;       /* alpha in delta = direction * exp(magnitude*alpha) * beta; paper: 0.01 */
  float step_mult;      /* beta in the same formula; paper: 0.01 */
  uint32_t lstm_hidden; /* VeLO only: LSTM width H_L (1..1024) */
  uint32_t n_bank;      /* VeLO only: number K of weight-bank rows (1..1024) */
  uint32_t apply_kernel; /* lopt_apply_kernel; 0 = automatic */
  uint32_t groups;      /* tensor groups of the two-stream pipeline, 1..16 (1 = every pass over the whole list, one after
                           the other, on the caller's stream); 0 = by list size */
  uint32_t state_pass;  /* lopt_state_pass; 0 = automatic */
} lopt_config;

typedef struct {
  uint32_t ndim; /* squeezed rank of the original tensor (>= 1) */
  int64_t rows;  /* m */
  int64_t cols;  /* n */
} lopt_tensor_desc;

/* Fill *cfg with the defaults for `kind`: decays {0.9,0.99,0.999}, 0.999, {0.9,0.99,0.999};
 * eps_acc 1e-16; eps_norm 1e-30; alpha = beta = 0.01; hidden 32 (small_fc_lopt) or 4 (VeLO);
 * lstm_hidden 512, n_bank 256; apply_kernel, groups and state_pass automatic. Returns LOPT_EINVAL for a null cfg or unknown kind. */
lopt_status lopt_default_config(uint32_t kind, lopt_config* cfg);

/* Number of floats lopt_create expects in weights_host for this configuration, 0 if the
 * configuration is invalid.
 *   small_fc_lopt: W1[39,H] b1[H] W2[H,H] b2[H] W3[H,2] b3[2]            (row-major; MLP of the
 *                  pseudocode of Kernel 2: Linear1, ReLU, Linear2, ReLU, Linear3)
 *   VeLO:          Wx[48,4H_L] Wh[H_L,4H_L] Wg[H_L,4H_L] b[4H_L] Wa[H_L,K] ba[K] ws[H_L] bs[1] B[K,P]
 *                  with P = 29H + H + H*H + H + 2H + 2; gate order i,f,g,o; Wg multiplies the
 *                  cross-tensor input, (ws, bs) is the step-size head; row q of B is a
 *                  flattened per-element MLP in the small_fc_lopt order with 29 inputs. */
size_t lopt_weights_count(const lopt_config* cfg);

/* Create a context. weights_host (n_weights floats) is copied to the current HIP device
 * before returning and may be freed afterwards. *out is set only on LOPT_OK.
 * Errors: LOPT_EINVAL (null, struct_size, hidden/lstm_hidden/n_bank out of range, decay
 * outside [0,1), negative eps), LOPT_ESTATE (n_weights != lopt_weights_count), LOPT_ENOMEM,
 * LOPT_EHIP.
 * Kernel and launch-plan selection is per context: cfg->apply_kernel, cfg->groups and cfg->state_pass. Where a field
 * is 0 (automatic), the environment may set it for experiments without touching the caller's code:
 *   LOPT_APPLY = auto | valu | mfma_f32 | mfma_f16s     LOPT_GROUPS = 0..16     LOPT_STATE_PASS = auto | stats | apply
 * Any other value of these, in the field or in the environment, is refused with LOPT_EINVAL. */
lopt_status lopt_create(const lopt_config* cfg, const float* weights_host, size_t n_weights,
                        lopt_ctx** out);

/* Free the context and its device memory. Null is ignored. The caller must make sure no
 * work enqueued through this context is still running. */
void lopt_destroy(lopt_ctx* ctx);

/* Sizes, in bytes, of each tensor's state blob (per_tensor_bytes[n]) and of the scratch
 * workspace one lopt_step over this list needs. Either output pointer may be null.
 *
 * State blob layout (fp32; pad4(x) = x rounded up to a multiple of 4 floats, N = rows*cols):
 *   M_1 | M_2 | M_3 | V       four sections of pad4(N) floats, row-major like the tensor
 *   r_1 | r_2 | r_3           three sections of pad4(rows) floats (Adafactor row accumulators)
 *   c_1 | c_2 | c_3           three sections of pad4(cols) floats (column accumulators)
 *   h | c_lstm                VeLO only: two sections of pad4(H_L) floats (LSTM state)
 * The blob is plain data: a checkpoint is a copy of it. The workspace holds nothing that
 * must survive from one call to the next. */
lopt_status lopt_state_bytes(const lopt_ctx* ctx, size_t n, const lopt_tensor_desc* descs_host,
                             size_t* per_tensor_bytes, size_t* workspace_bytes);

/* Zero every state blob (zero-initialised accumulators, no bias correction). state_host is
 * a host array of n device pointers. workspace is unused and may be null. */
lopt_status lopt_init_state(lopt_ctx* ctx, size_t n, const lopt_tensor_desc* descs_host,
                            void* const* state_host, void* workspace, void* hip_stream);

/* One optimizer step over the whole list (the paper's Optimizer.step):
 *   1. M_i <- beta_i M_i + (1-beta_i) g;  V <- beta_4 V + (1-beta_4) g^2;
 *      r_k <- beta r_k + (1-beta) row_mean(g^2);  c_k <- beta c_k + (1-beta) col_mean(g^2)
 *   2. per tensor and feature f: s_f = mean over the tensor of feature_f^2
 *   3. (VeLO) one LSTM-cell step per tensor on u = [0.05 ln(s_f + 1e-30), tanh(step/x), one-hot(ndim),
 *      loss features]: gates z = u Wx + h Wh + hbar Wg + b, where hbar is the mean over the tensors of
 *      THIS call's list of their LSTM outputs h before the step (zero state: zeros); per-tensor MLP
 *      weights theta = (h' W_a + b_a) B and step-size multiplier lam = exp(h' . ws + bs)
 *      (small_fc_lopt: lam = 1)
 *   4. per element: x_f = feature_f / sqrt(s_f + eps_norm) (time features un-normalized),
 *      (direction, magnitude) = MLP(x), delta = lam * direction * exp(alpha*magnitude) * beta,
 *      p <- p - lr * (delta + weight_decay * p)
 * params_host, grads_host, state_host: host arrays of n device pointers (grads are read only).
 * step: number of updates already applied (0 on the first call), must be >= 0.
 * lr, weight_decay: finite. The call is asynchronous with respect to the host.
 * Errors: LOPT_EINVAL, LOPT_ESHAPE, LOPT_ENOMEM, LOPT_EHIP (see lopt_status). */
lopt_status lopt_step(lopt_ctx* ctx, size_t n, const lopt_tensor_desc* descs_host,
                      float* const* params_host, const float* const* grads_host,
                      void* const* state_host, void* workspace, int64_t step, float lr,
                      float weight_decay, void* hip_stream);

/* The loss value that goes with the gradients of the following steps (the paper's VeLO usage passes the
 * current loss to Optimizer.step; artifact appendix, "Basic Usage"). Host scalar, finite; used by every
 * lopt_step / lopt_step_static through this context until set again; 0 (no loss features) when never
 * set. small_fc_lopt ignores it. Errors: LOPT_EINVAL (null ctx, non-finite loss). */
lopt_status lopt_set_loss(lopt_ctx* ctx, float loss);

/* lopt_step for callers that cannot allocate device memory: code under HIP graph capture, tight serving
 * loops, harnesses that forbid hipMalloc. Same arguments, semantics and results as lopt_step, minus the
 * workspace: the device tables and the workspace live in a fixed array of LOPT_STATIC_SCRATCH_BYTES bytes
 * that is part of the library's device image (every GPU the library runs on holds its own copy until the
 * process ends; its address on a device is resolved once, in lopt_create). The call makes no hipMalloc,
 * hipFree, hipHostMalloc or event creation: tables are staged through the pinned buffer every context is
 * created with (4 MiB).
 *   - A list whose tables plus workspace exceed the array, or whose tables exceed the staging buffer, is
 *     refused with LOPT_ELIMIT before anything is launched (the message gives both sizes). The ViT-B/16
 *     parameter set (152 tensors, 86.6 M elements) needs about 12 MiB.
 *   - Nothing in the array has to start at zero (the apply pass's tile counters are cleared inside every
 *     step) and nothing in it survives a call: all calls on one GPU, through any context, share it. Calls
 *     that overlap on one GPU (different streams, different host threads) race; calls ordered on one
 *     stream are safe, and a context re-sends its tables after another context has used the array.
 *   - Per-pass timing (lopt_profile_enable) does not apply to this entry point. */
#define LOPT_STATIC_SCRATCH_BYTES (64u << 20)
lopt_status lopt_step_static(lopt_ctx* ctx, size_t n, const lopt_tensor_desc* descs_host,
                             float* const* params_host, const float* const* grads_host,
                             void* const* state_host, int64_t step, float lr, float weight_decay,
                             void* hip_stream);

/* Byte offsets, inside the workspace, of each tensor's feature statistics s_f as left by the
 * last lopt_step over this list: d floats per tensor (d = 28 for small_fc_lopt, whose time
 * features are not normalized; 29 for VeLO), in the feature order
 *   0 g | 1 p | 2-4 M_i | 5 V | 6-8 M_i/sqrt(V) | 9 1/sqrt(V) | 10-12 g*fac_k | 13-15 r_k |
 *   16-18 c_k | 19-21 1/sqrt(r_k) | 22-24 1/sqrt(c_k) | 25-27 M_k*fac_k | 28 clip(g,-0.1,0.1)
 * with fac_k = sqrt(mean(r_k) / (r_k c_k^T)). For inspection and tests. */
lopt_status lopt_stats_offsets(const lopt_ctx* ctx, size_t n, const lopt_tensor_desc* descs_host,
                               size_t* offsets_bytes);

/* Per-pass timing for benchmarks. lopt_step is a fixed sequence of LOPT_N_PASSES kernel launches
 * (a pass that a configuration does not use records zero time):
 *   0 rowcol_sums  1 rc_update  2 accum_stats  3 finalize  4 velo_lstm  5 velo_head  6 apply
 * With profiling enabled, lopt_step runs every pass over the whole list on the caller's stream (no
 * tensor groups, no second stream) and brackets every launch with HIP events on that stream.
 * lopt_profile_read waits for the recorded events, adds up the elapsed milliseconds per pass over
 * all steps since the last read (ms_per_pass[LOPT_N_PASSES], may not be null), stores the number of
 * steps in *n_steps (may be null) and clears the record. lopt_pass_name returns a static string,
 * NULL for an index out of range. Profiling is off by default; it does not change any result. */
#define LOPT_N_PASSES 7
lopt_status lopt_profile_enable(lopt_ctx* ctx, int on);
lopt_status lopt_profile_read(lopt_ctx* ctx, double* ms_per_pass, uint64_t* n_steps);
const char* lopt_pass_name(int pass);

/* Message for the last non-OK status returned through this context ("" if none). With a
 * null ctx: the message of the last failed lopt_create / lopt_default_config on this thread. */
const char* lopt_last_error(const lopt_ctx* ctx);

#ifdef __cplusplus
}
#endif
#endif /* LOPT_H */
