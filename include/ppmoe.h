/* ppmoe.h -- C ABI of libppmoe.so: the MoE-layer forward of Pipeline MoE (PPMoE) on one device's
 * share of a tensor-parallel group, as hand-written HIP kernels for gfx950 (MI355X).
 *
 * The path is Algorithm 1 of the paper without its closing all-reduce:
 *   gate (linear map, softmax, top-k)  ->  tensor-index-slicing dispatch  ->  local expert FFNs
 *   ->  gate-weighted combine into the zero-initialised partial output [T, d].
 *
 * Conventions that hold for every function below
 *   - Every data pointer is a DEVICE pointer owned by the caller, 16-byte aligned, row-major and
 *     contiguous.  Only `const moe_config*` and `stage_events` arrays are HOST pointers.
 *   - `stream` is a hipStream_t passed as void* (NULL = the null stream).  Work is enqueued
 *     asynchronously; nothing here allocates or frees device memory.  Results are valid once the
 *     caller has synchronised the stream.  The calls that SYNCHRONISE the stream are: moe_init;
 *     moe_ffn_check; moe_ffn_clock; moe_event_elapsed_ms (on its event); and, once per device and only if moe_init
 *     has not been called for that device, the first expert-FFN call (moe_expert_ffn, _up, _down,
 *     moe_layer_forward, moe_expert_ffn_backward) with bf16/fp16 input -- unless that call is made
 *     under stream capture, where nothing synchronises (see moe_init).
 *   - Return value: MOE_OK (0) or a negative moe_status.  Arguments are validated on the host
 *     before anything is launched; on error nothing has been enqueued.
 *   - Weights are stored [out, in] (the contraction index is contiguous):
 *     Wg[E, d], W1[N, F, d] (the paper's A_i transposed), W2[N, d, F] (B_i transposed).
 *   - in_dtype is the type of x, Wg, W1, W2, x_sliced, H, y_sliced; out_dtype the type of `out`.
 *     Supported pairs: (F32, F32), (BF16, BF16), (BF16, F32), (F16, F16), (F16, F32) -- F16 is IEEE
 *     half precision, the paper's own training precision (Section 4.1).  Logits, softmax and gate
 *     weights are always float32 (the paper keeps the gating module in float32, Section 4.1); GEMMs
 *     accumulate in float32 and round to nearest even when they store a 16-bit type.
 *   - Shapes: T >= 0 tokens, d and F multiples of 8, 1 <= top_k <= E <= 256, top_k <= 8,
 *     0 <= local_begin, local_begin + local_count <= E, local_count >= 1, k*T < 2^31.
 *   - Inputs are assumed finite.  With NaN logits the pick order is unspecified.
 */
#ifndef PPMOE_H
#define PPMOE_H

#include <stddef.h>
#include <stdint.h>

#ifdef __cplusplus
extern "C" {
#endif

typedef enum {
  MOE_OK = 0,
  MOE_ERR_NULL = -1,      /* a required pointer is NULL                              */
  MOE_ERR_SHAPE = -2,     /* a size violates the limits listed above                 */
  MOE_ERR_DTYPE = -3,     /* unsupported (in_dtype, out_dtype) pair                  */
  MOE_ERR_ALIGN = -4,     /* a device pointer is not 16-byte aligned                 */
  MOE_ERR_WORKSPACE = -5, /* workspace_bytes smaller than moe_workspace_bytes(cfg)   */
  MOE_ERR_HIP = -6        /* a HIP runtime call (launch, event record) failed        */
} moe_status;

typedef enum { MOE_F32 = 0, MOE_BF16 = 1, MOE_F16 = 2 } moe_dtype;

/* Problem statement of one MoE layer on one device (Sections 3.3.1-3.3.3):
 * T = b*s token embeddings of size d = h, E experts in the tensor-parallel group of which this
 * device holds the contiguous block [local_begin, local_begin + local_count), a top_k gating
 * schedule, and an optional capacity limit (PPMoE itself runs without one, Section 4.1). */
typedef struct {
  int32_t T, d, F;          /* tokens, hidden size, FFN inner size                             */
  int32_t E, top_k;         /* experts in the group, picks per token                           */
  int32_t local_begin, local_count;
  float capacity_factor;    /* <= 0: no limit; else every expert keeps the first
                               C = ceil(capacity_factor * top_k * T / E) assignments of its
                               queue (ascending t*top_k + j) and drops the rest              */
  int32_t renorm_topk;      /* 1: gate weights are divided by their sum over the k picks       */
  int32_t in_dtype;         /* moe_dtype                                                       */
  int32_t out_dtype;        /* moe_dtype                                                       */
} moe_config;

/* Stages of the fused call, in launch order; moe_layer_forward records stage_events[i] before
 * stage i and stage_events[MOE_NUM_STAGES] after the last one. */
enum {
  MOE_STAGE_GATE = 0,     /* router GEMM + softmax + top-k                         */
  MOE_STAGE_PERMUTE = 1,  /* histogram, scan, stable positions                     */
  MOE_STAGE_SLICE = 2,    /* row gather into x_sliced                              */
  MOE_STAGE_FFN_UP = 3,   /* grouped GEMM  H = GeLU(x_sliced W1^T)                 */
  MOE_STAGE_FFN_DOWN = 4, /* grouped GEMM  y_sliced = H W2^T                       */
  MOE_STAGE_COMBINE = 5,  /* gate-weighted gather into out                         */
  MOE_NUM_STAGES = 6
};

/* Set-up -------------------------------------------------------------------------------------- */

/* One-time set-up of the CURRENT device for the expert GEMMs: kernel attributes and the placement
 * check of the persistent blocks (a probe kernel is launched on `stream` and waited for: this call
 * SYNCHRONISES the stream, so it must not be made under stream capture).  Calling it is optional
 * but recommended before the first layer call: without it the first expert-FFN call on the device
 * does the same work, synchronising once; and if that first call is being captured into a graph it
 * cannot run the check, so it (and every later launch until the check has run outside a capture)
 * hands partial sums over with device-scope fences, which is correct on any placement but slower.
 * Idempotent; cheap after the first call. */
int moe_init(void* stream);

/* Diagnostic switches (process-wide, take effect at the next launch; not needed in normal use).
 *   MOE_OPT_HANDOVER_DEVICE_SCOPE  value != 0: partial sums of output tiles cut between compute
 *        units are always handed over with device-scope fences, whatever the placement check found
 *        (the path a device with another block placement would take); 0: back to automatic.
 *   MOE_OPT_HANDOVER_SPIN_LIMIT    how many times a compute unit polls for another one's partial
 *        sums before it gives up and computes the missing part of the tile itself (default 131072;
 *        0: never wait, always compute it itself).  The output is complete either way.
 * Returns MOE_ERR_SHAPE for an unknown option or a value outside [0, 2^31). */
enum { MOE_OPT_HANDOVER_DEVICE_SCOPE = 1, MOE_OPT_HANDOVER_SPIN_LIMIT = 2 };
int moe_set_option(int option, int64_t value);

/* Host-only helpers ------------------------------------------------------------------------- */

/* Text for a moe_status value (static storage, never NULL). */
const char* moe_status_string(int status);

/* Per-expert queue limit C for this configuration, or -1 when capacity_factor <= 0.
 * Computed in double precision exactly as ceil((double)cf * top_k * T / E). */
int64_t moe_capacity(const moe_config* cfg);

/* Upper bound on packed rows: top_k*T without a capacity limit, else
 * min(top_k*T, local_count*C).  Buffers indexed by packed row (perm, x_sliced, H, y_sliced) must
 * hold this many rows. */
int64_t moe_max_rows(const moe_config* cfg);

/* Bytes of scratch the largest consumer (moe_layer_forward) needs.  0 on an invalid config. */
size_t moe_workspace_bytes(const moe_config* cfg);

/* Bytes of scratch moe_slice_dispatch needs (per-segment counters of the permutation); never more
 * than moe_workspace_bytes(cfg).  0 on an invalid config. */
size_t moe_dispatch_workspace_bytes(const moe_config* cfg);

/* Bytes of scratch the expert-FFN calls need (partial sums of output tiles whose k range is cut
 * between compute units); never more than moe_workspace_bytes(cfg).  0 on an invalid config. */
size_t moe_ffn_workspace_bytes(const moe_config* cfg);

/* Stage entry points ------------------------------------------------------------------------ */

/* Gating module (Section 3.3.3; Algorithm 1: wg, softmax, gate_function).
 *   logits[t, e] = sum_i x[t, i] * Wg[e, i] + bias[e]           (float32 accumulation)
 *   p = softmax over all E experts; the top_k largest logits are picked, equal logits going to the
 *   lower expert index; expert_idx[t, :] lists the picks in descending-logit order and
 *   gate_w[t, j] = p[t, expert_idx[t, j]], divided by its sum over j when cfg->renorm_topk.
 * x [T, d] in_dtype; Wg [E, d] in_dtype; bias [E] float32 or NULL.
 * logits_in [T, E] float32 or NULL: when given, x/Wg/bias are ignored (may be NULL) and these
 * logits are used verbatim.  logits_out [T, E] float32 or NULL receives the logits used.
 * expert_idx [T, top_k] int32 and gate_w [T, top_k] float32 are written in full. */
int moe_gate(const moe_config* cfg, const void* x, const void* Wg, const float* bias,
             const float* logits_in, float* logits_out, int32_t* expert_idx, float* gate_w,
             void* stream);

/* Auxiliary load-balance loss, the second value Algorithm 1 returns ("l_aux").  The paper takes it
 * from GShard (Section 4.1) and prints no formula; this is the GShard form:
 *   l_aux = E * sum_e mean_prob[e] * first_counts[e] / T,
 *   mean_prob[e]    = mean over the T tokens of softmax(logits)[t, e]      (float32),
 *   first_counts[e] = number of tokens whose first pick expert_idx[t, 0] is e (also when top_k > 1;
 *                     before any capacity drop).
 * logits [T, E] float32 (what moe_gate wrote to logits_out); expert_idx [T, top_k] int32.
 * l_aux: one float32 in device memory; mean_prob [E] float32 and first_counts [E] int32 in device
 * memory, either may be NULL.  T == 0 gives zeros.  Sums have a fixed order (bitwise reproducible).
 * workspace: device memory of at least moe_aux_workspace_bytes(cfg) bytes, overwritten. */
size_t moe_aux_workspace_bytes(const moe_config* cfg);
int moe_aux_loss(const moe_config* cfg, const float* logits, const int32_t* expert_idx, float* l_aux,
                 float* mean_prob, int32_t* first_counts, void* workspace, size_t workspace_bytes,
                 void* stream);

/* Tensor-index-slicing dispatch (Sections 3.3.1 and 3.3.3, the index selection that replaces the
 * first all-to-all; Algorithm 1: sliced_inputs).  Assignment id a = t*top_k + j.  The queue of an
 * expert is every assignment that picked it, in ascending a; with a capacity limit only the first
 * C are kept.  The kept queues of the local experts are packed end to end in ascending expert
 * order (the paper's worked example: order 2,3,1,2,0,3,2,0 gives [4,7] [2] [0,3,6] [1,5]).
 *   counts [local_count]        kept queue lengths
 *   offsets [local_count + 1]   exclusive prefix sum of counts
 *   perm [moe_max_rows]         perm[r] = assignment id in packed row r, r < offsets[local_count]
 *   inv_perm [T, top_k]         packed row of (t, j), or -1 when dropped or not local
 *   x_sliced [moe_max_rows, d]  x_sliced[r, :] = x[perm[r] / top_k, :]; NULL skips the row copy
 * Rows at or beyond offsets[local_count] of perm and x_sliced are left untouched.
 * workspace: at least moe_dispatch_workspace_bytes(cfg) bytes of device scratch. */
int moe_slice_dispatch(const moe_config* cfg, const void* x, const int32_t* expert_idx,
                       int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                       void* x_sliced, void* workspace, size_t workspace_bytes, void* stream);

/* moe_slice_dispatch for callers that cannot allocate device memory or bring a workspace: code under
 * HIP graph capture, tight serving loops, harnesses that forbid hipMalloc.  Same arguments, results
 * and kernels as moe_slice_dispatch, but the permutation's per-segment counters live in a fixed
 * array of MOE_STATIC_SCRATCH_BYTES (4 MiB) of device memory inside the library (one copy on
 * every device it runs on, held until the process ends) instead of a caller's workspace.  It
 * allocates and frees nothing.  Limit: moe_dispatch_workspace_bytes(cfg) must not exceed
 * MOE_STATIC_SCRATCH_BYTES, i.e. (2 * ceil(top_k*T / 64) + 1) * local_count * 4 bytes <= 4 MiB
 * (top_k*T up to about 4 million assignments with 8 local experts); beyond that the call returns
 * MOE_ERR_WORKSPACE and launches nothing.  Every call on a device shares that device's array, and
 * the array keeps the last call's contents (the kernels overwrite every counter they read, nothing
 * needs clearing): calls that overlap in time on one device -- different streams -- race; order
 * them on one stream or with events. */
#define MOE_STATIC_SCRATCH_BYTES (4u << 20)
int moe_slice_dispatch_static(const moe_config* cfg, const void* x, const int32_t* expert_idx,
                              int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                              void* x_sliced, void* stream);

/* The row gather of moe_slice_dispatch alone (Algorithm 1: hidden_states.index_select), from index
 * lists already built:  x_sliced[r, :] = x[perm[r] / top_k, :]  for r < offsets[local_count].
 * x [T, d] in_dtype; perm [moe_max_rows] int32 and offsets [local_count + 1] int32 as written by
 * moe_slice_dispatch; x_sliced [moe_max_rows, d] in_dtype (rows beyond offsets[local_count] are
 * left untouched). */
int moe_slice_rows(const moe_config* cfg, const void* x, const int32_t* perm, const int32_t* offsets,
                   void* x_sliced, void* stream);

/* Local experts (Section 3.3.2: the N experts of a device; FFN of Section 3.1.3, GeLU(X A) B with
 * the tanh form of GeLU and no bias), evaluated as two grouped GEMMs over the packed rows:
 *   H[r, :]        = GeLU(x_sliced[r, :] . W1[i]^T)   for offsets[i] <= r < offsets[i+1]
 *   y_sliced[r, :] = H[r, :] . W2[i]^T
 * x_sliced [rows, d], H [rows, F] (scratch the caller provides), y_sliced [rows, d], all in_dtype,
 * rows = moe_max_rows(cfg); offsets is the device array moe_slice_dispatch wrote (never read on
 * the host).  Rows at or beyond offsets[local_count] are not written.
 * workspace: at least moe_ffn_workspace_bytes(cfg) bytes of device scratch; calls that share a
 * workspace must be ordered on one stream.
 * moe_expert_ffn_up / _down run one of the two GEMMs each; moe_expert_ffn runs both. */
int moe_expert_ffn_up(const moe_config* cfg, const void* x_sliced, const int32_t* offsets,
                      const void* W1, void* H, void* workspace, size_t workspace_bytes,
                      void* stream);
int moe_expert_ffn_down(const moe_config* cfg, const void* H, const int32_t* offsets,
                        const void* W2, void* y_sliced, void* workspace, size_t workspace_bytes,
                        void* stream);
int moe_expert_ffn(const moe_config* cfg, const void* x_sliced, const int32_t* offsets,
                   const void* W1, const void* W2, void* H, void* y_sliced, void* workspace,
                   size_t workspace_bytes, void* stream);

/* Backward of the local experts (Section 3.2, footnote to Eq. 1: the backward pass costs about twice the
 * forward; Section 3.3.4: it exchanges the same tensors; the paper prints no backward algorithm, this
 * is the chain rule of moe_expert_ffn).  With U = x_sliced W1[i]^T, H = GeLU(U), y_sliced = H W2[i]^T
 * for the packed rows offsets[i] <= r < offsets[i+1] of expert i, and dY = dLoss/dy_sliced:
 *   dX_sliced[r, :] = (dY[r, :] W2[i] * GeLU'(U[r, :])) W1[i]            [rows, d]  in_dtype
 *   dW1[i]          = sum_r (dY[r, :] W2[i] * GeLU'(U[r, :]))^T x_sliced[r, :]   [F, d]  float32
 *   dW2[i]          = sum_r dY[r, :]^T H[r, :]                                     [d, F]  float32
 * (the weight gradients in the weights' own [out, in] layout, overwritten, not accumulated; an expert
 * without rows gets zeros).  U is recomputed from x_sliced, so the forward need keep nothing.
 * in_dtype BF16 or F16 only (MOE_ERR_DTYPE otherwise).  x_sliced, dY, dX_sliced: [moe_max_rows, d];
 * rows at or beyond offsets[local_count] are neither read nor written.
 * workspace: at least moe_ffn_backward_workspace_bytes(cfg) bytes of device scratch (three
 * [moe_max_rows, F] buffers, the expert GEMM's own scratch and, with at most 16 local experts, 8192 * d
 * bytes per local expert of float32 partial sums for the experts' last rows of dX_sliced); the first
 * expert-FFN call of a device may synchronise once, see moe_init. */
size_t moe_ffn_backward_workspace_bytes(const moe_config* cfg);
int moe_expert_ffn_backward(const moe_config* cfg, const void* x_sliced, const int32_t* offsets,
                            const void* W1, const void* W2, const void* dY, void* dX_sliced, float* dW1,
                            float* dW2, void* workspace, size_t workspace_bytes, void* stream);

/* Backward of the whole layer (the chain rule of moe_layer_forward with the picks -- top-k and capacity
 * drops -- held fixed; Section 3.2, footnote to Eq. 1; Section 3.3.4: in a tensor-parallel group the
 * backward exchanges the same tensors as the forward, i.e. one all-reduce of dx, outside this call).
 * Given d_out = dLoss/d(out) [T, d] in out_dtype, with (t, j) -> r the kept local assignments:
 *   dY[r, :]       = gate_w[t, j] * d_out[t, :]
 *   d_gate_w[t, j] = <d_out[t, :], y_sliced[r, :]>   (0 for dropped or non-local picks)
 *   dlogits        = d_gate_w through the (renormalised) top-k weights and the softmax
 *   dx[t, :]       = sum over kept local (t, j) of dX_sliced[r, :]  +  dlogits[t, :] Wg     [T, d]  in_dtype
 *   dWg            = dlogits^T x   [E, d] float32;   dbias = column sums of dlogits   [E] float32 or NULL
 *   dW1, dW2       as in moe_expert_ffn_backward
 * Everything is this device's partial sum: over the devices of a tensor-parallel group dx, dWg and
 * dbias add up to the gradients of the whole layer (a pick that is local elsewhere contributes there).
 * The gradient of l_aux is not included.  The routing is recomputed from x and Wg, so nothing has to be
 * kept from the forward call.  in_dtype BF16 or F16 only.
 * workspace: at least moe_layer_backward_workspace_bytes(cfg) bytes of device scratch. */
size_t moe_layer_backward_workspace_bytes(const moe_config* cfg);
int moe_layer_backward(const moe_config* cfg, const void* x, const void* Wg, const float* bias, const void* W1,
                       const void* W2, const void* d_out, void* dx, float* dWg, float* dbias, float* dW1,
                       float* dW2, void* workspace, size_t workspace_bytes, void* stream);

/* Forward and backward of a training step that keeps the forward's intermediates instead of computing
 * them again (Section 3.2, footnote to Eq. 1: the backward then costs the four gradient products,
 * twice the forward's two).
 * moe_layer_forward_train is moe_layer_forward_aux (same `out`, l_aux, mean_prob, first_counts) that
 * also leaves in `saved` (>= moe_layer_saved_bytes(cfg) bytes of device memory, 16-byte aligned) the
 * routing (picks, gate weights, offsets, permutation and its inverse, the float32 logits), the
 * sliced tokens, U = x_sliced A and H = GeLU(U), both in in_dtype.  The activation is applied by a
 * pass over the stored U, so H, and with it `out`, is rounded once more than in moe_layer_forward.
 * moe_layer_backward_saved computes what moe_layer_backward computes (same outputs, same formulas)
 * from `saved` as the forward call with the same cfg, x, Wg, bias, W1 and W2 left it; it reads `saved`
 * and does not change it.  Neither call allocates or synchronises: a step can be captured into a
 * HIP graph (after one eager call, which sets kernel attributes).  workspace: moe_workspace_bytes(cfg) for the forward,
 * moe_layer_backward_workspace_bytes(cfg) for the backward.  in_dtype BF16 or F16 only
 * (MOE_ERR_DTYPE otherwise; moe_layer_saved_bytes returns 0). */
size_t moe_layer_saved_bytes(const moe_config* cfg);
int moe_layer_forward_train(const moe_config* cfg, const void* x, const void* Wg, const float* bias,
                            const void* W1, const void* W2, void* out, float* l_aux, float* mean_prob,
                            int32_t* first_counts, void* saved, size_t saved_bytes, void* workspace,
                            size_t workspace_bytes, void* stream);
int moe_layer_backward_saved(const moe_config* cfg, const void* x, const void* Wg, const void* W1,
                             const void* W2, const void* d_out, const void* saved, size_t saved_bytes, void* dx,
                             float* dWg, float* dbias, float* dW1, float* dW2, void* workspace,
                             size_t workspace_bytes, void* stream);

/* Health of the expert-FFN calls that used `workspace` since the last check.  When an output tile
 * is cut between compute units, the partial sums are handed over through the workspace with a
 * bounded wait.  The persistent kernel expects one block per compute unit to be resident at once,
 * i.e. the device not to be shared with another stream's kernels while it runs; if a block starts
 * late, the unit waiting for its partial sums gives up after the spin limit and computes that part
 * of the tile itself.  The OUTPUT IS COMPLETE AND CORRECT EITHER WAY (only the float32 summation
 * order of that tile differs from an undisturbed run, and time was lost); this call tells whether
 * it happened.  It copies the kernel's word to the host (it SYNCHRONISES the stream) and sets
 * *status (host) to 0: every hand-over went through; 1: at least one partial sum did not arrive
 * within the spin limit; 2: writer and reader of a partial sum ran on different XCDs although the
 * placement check at set-up said they would not (the reader then recomputed as in case 1).  A
 * reported word is cleared.  layer_workspace != 0: `workspace` is the one given to
 * moe_layer_forward; 0: the one given to moe_expert_ffn / _up / _down. */
int moe_ffn_check(const moe_config* cfg, const void* workspace, int layer_workspace,
                  int32_t* status, void* stream);

/* Combine (Sections 3.3.1/3.3.3, the index assignment that replaces the second all-to-all;
 * Algorithm 1: zeros_like + placement):
 *   out[t, :] = sum over j ascending with inv_perm[t, j] >= 0 of gate_w[t, j] * y_sliced[inv_perm[t, j], :]
 * accumulated in float32 and rounded once to out_dtype; rows with no kept local pick are +0.
 * Every row of out [T, d] is written exactly once (no atomics, no separate zero fill). */
int moe_combine(const moe_config* cfg, const void* y_sliced, const int32_t* inv_perm,
                const float* gate_w, void* out, void* stream);

/* The whole layer (Algorithm 1 up to, not including, reduce_from_tensor_parallel_region): the six
 * stages above on one stream with no host round trip.  Intermediates live in `workspace`
 * (>= moe_workspace_bytes(cfg)); `out` [T, d] out_dtype is the partial sum this device would
 * contribute to the all-reduce.  Where moe_layer_fuses(cfg) says so, the slice and the combine are
 * carried out by the loads of the first and the stores of the second expert GEMM and x_sliced /
 * y_sliced are not written; everything else in the workspace is.
 * stage_events: NULL, or a HOST array of MOE_NUM_STAGES + 1 hipEvent_t handles (as void*) that are
 * recorded on `stream` around the stages, for timing. */
int moe_layer_forward(const moe_config* cfg, const void* x, const void* Wg, const float* bias,
                      const void* W1, const void* W2, void* out, void* workspace,
                      size_t workspace_bytes, void* const* stage_events, void* stream);

/* moe_layer_forward that also returns the second value of Algorithm 1, the auxiliary balance loss
 * (formula and conventions: see moe_aux_loss), without a second pass over the tokens: the gating
 * kernel adds up the softmax probabilities and the first picks per expert while it scores the tokens
 * (per block of tokens, in token order) and the permutation's scan launch adds the blocks' sums in
 * order, so the loss is bitwise reproducible and no [T, E] logits are written.  (float32 input, more
 * than 64 experts, or a router matrix too large for the LDS: the logits go through the workspace and
 * the kernels of moe_aux_loss run after the gate.)
 * l_aux: one float32 in DEVICE memory (4-byte aligned), or NULL for exactly moe_layer_forward;
 * mean_prob [E] float32 and first_counts [E] int32 in device memory, either may be NULL (both must be
 * NULL when l_aux is).  Everything else as moe_layer_forward. */
int moe_layer_forward_aux(const moe_config* cfg, const void* x, const void* Wg, const float* bias,
                          const void* W1, const void* W2, void* out, float* l_aux, float* mean_prob,
                          int32_t* first_counts, void* workspace, size_t workspace_bytes,
                          void* const* stage_events, void* stream);

/* Which stages moe_layer_forward folds into the expert GEMMs for `cfg` (bf16 / fp16 input, d a
 * multiple of 64): a mask of
 *   MOE_FUSE_SLICE    the first GEMM reads the token rows through the permutation (Algorithm 1's
 *                     index selection done by its loads): x_sliced is not written;
 *   MOE_FUSE_COMBINE  (output of the input's 16-bit type, F a multiple of 64) the second GEMM applies the
 *                     gate weight and stores straight into `out` every packed row that is its token's
 *                     only kept local pick (the placement of the expert outputs done by its stores).
 *                     top_k == 1: that is every row, y_sliced is not written, and rows of `out`
 *                     without a kept local pick are zeroed by a kernel of their own.  top_k >= 2: rows
 *                     of tokens with several kept local picks are still written to y_sliced and
 *                     summed by the combine kernel, which leaves the placed rows alone; the other
 *                     rows of y_sliced are not written.
 * 0: every intermediate is written. */
enum { MOE_FUSE_SLICE = 1, MOE_FUSE_COMBINE = 2 };
int moe_layer_fuses(const moe_config* cfg);

/* Where moe_layer_forward keeps its intermediates inside `workspace` (byte offsets), so a caller
 * can inspect them after a run.  Any pointer may be NULL. */
typedef struct {
  size_t expert_idx, gate_w, counts, offsets, perm, inv_perm, x_sliced, H, y_sliced, scratch, gemm;
  size_t logits, aux;   /* scratch of the balance loss (moe_layer_forward_aux)                   */
} moe_workspace_layout;
int moe_workspace_offsets(const moe_config* cfg, moe_workspace_layout* layout);

/* Plain device-to-device copy of `bytes` bytes (a multiple of 16) by a kernel that reads and writes
 * every byte exactly once.  Not part of the layer: it is the reference of known traffic against
 * which hardware byte counters (FETCH_SIZE, WRITE_SIZE) are calibrated when profiling. */
int moe_copy_bytes(const void* src, void* dst, size_t bytes, void* stream);

/* Register-resident bf16 MFMA loop with the grouped GEMM's launch shape (one block of four
 * wavefronts per CU, 16 accumulator blocks of 32x32x16 per wavefront) and no memory traffic: the
 * empirical ceiling of the matrix cores, against which the GEMMs' TFLOP/s can be read next to the
 * published peak.  Not part of the layer.  `iters` loop iterations of 16 MFMAs per wavefront;
 * `random_operands` != 0 fills the operand registers with pseudo-random values in [-1, 1) (the
 * clock then settles lower, under the power limit, than with constant operands); `sink`: device
 * memory for 65536 floats (overwritten); `*flops` (host) receives the flop count of the launch. */
int moe_mfma_probe(int64_t iters, int random_operands, float* sink, double* flops, void* stream);

/* What clock the matrix-core kernels ran at.  The fast path of the grouped GEMMs (Section 3.3.2) leaves
 * in its scratch the shader-clock and wall-clock counters its first block read at its start and its
 * end; this reads them back for the LAST such launch on `workspace` (the one given to moe_expert_ffn_*,
 * or, layer_workspace != 0, to moe_layer_forward) and returns the shader clock in GHz and the
 * block's lifetime in microseconds (both 0 if no fast-path launch has used the workspace).  A
 * measurement helper: under load the clock settles well below the 2.4 GHz the published peak is
 * quoted at, and a fraction of that peak has to be read with this beside it.  Synchronises `stream`. */
int moe_ffn_clock(const moe_config* cfg, const void* workspace, int layer_workspace, double* shader_ghz,
                  double* kernel_us, void* stream);

/* Timing helpers: thin wrappers over hipEvent so a caller without HIP headers can time stages.
 * moe_event_elapsed_ms synchronises on `stop` before reading. */
int moe_event_create(void** event);
int moe_event_destroy(void* event);
int moe_event_record(void* event, void* stream);
int moe_event_elapsed_ms(void* start, void* stop, float* ms);

#ifdef __cplusplus
}
#endif
#endif /* PPMOE_H */
