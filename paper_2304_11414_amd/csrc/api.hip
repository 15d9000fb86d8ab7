// Host side of libppmoe.so: argument validation, workspace layout and the launch sequence of
// Algorithm 1 (without its closing all-reduce).  Nothing here allocates; what may synchronise is
// listed in ppmoe.h (moe_init, moe_ffn_check, moe_event_elapsed_ms, and the first expert-FFN call on
// a device that moe_init has not prepared).

#include <cmath>
#include <cstring>

#include "common.h"

using namespace ppmoe;

namespace {

constexpr size_t kAlign = 256;
inline size_t align_up(size_t v) { return (v + kAlign - 1) / kAlign * kAlign; }
inline bool misaligned(const void* p) { return (reinterpret_cast<uintptr_t>(p) & 15u) != 0; }
inline size_t elem_bytes(int dtype) { return is_16bit(dtype) ? 2 : 4; }

int check_config(const moe_config* c) {
  if (c == nullptr) return MOE_ERR_NULL;
  if (c->T < 0 || c->d <= 0 || c->F <= 0 || (c->d & 7) || (c->F & 7)) return MOE_ERR_SHAPE;
  if (c->E < 1 || c->E > kMaxExperts) return MOE_ERR_SHAPE;
  if (c->top_k < 1 || c->top_k > c->E || c->top_k > kMaxTopK) return MOE_ERR_SHAPE;
  if (c->local_begin < 0 || c->local_count < 1 || c->local_begin + c->local_count > c->E)
    return MOE_ERR_SHAPE;
  if (static_cast<int64_t>(c->T) * c->top_k >= (1ll << 31)) return MOE_ERR_SHAPE;
  const bool ok = (c->in_dtype == MOE_F32 && c->out_dtype == MOE_F32) ||
                  (is_16bit(c->in_dtype) && (c->out_dtype == c->in_dtype || c->out_dtype == MOE_F32));
  if (!ok) return MOE_ERR_DTYPE;
  if (!(c->capacity_factor == c->capacity_factor)) return MOE_ERR_SHAPE;  // NaN
  return MOE_OK;
}

int64_t capacity_of(const moe_config& c) {
  if (!(c.capacity_factor > 0.f)) return -1;
  double v = std::ceil(static_cast<double>(c.capacity_factor) * c.top_k * c.T / c.E);
  if (v > 2147483647.0) v = 2147483647.0;
  return static_cast<int64_t>(v);
}

int64_t max_rows_of(const moe_config& c) {
  const int64_t all = static_cast<int64_t>(c.T) * c.top_k;
  const int64_t cap = capacity_of(c);
  int64_t per_expert = c.T;  // an expert is picked at most once per token (Section 4.1: at most b*s)
  if (cap >= 0 && cap < per_expert) per_expert = cap;
  const int64_t by_expert = per_expert * c.local_count;
  return by_expert < all ? by_expert : all;
}

size_t dispatch_scratch_bytes(const moe_config& c) {
  int64_t segs = max_segments(c);
  if (segs < 1) segs = 1;
  return static_cast<size_t>(2 * segs + 1) * c.local_count * sizeof(int32_t);
}

// Scratch of the balance loss inside the layer's workspace: the per-segment partial sums the gating
// kernel leaves, or what the stand-alone loss kernels need, whichever is larger.
size_t aux_region_bytes(const moe_config& c) {
  const size_t fused = static_cast<size_t>(max_segments(c)) * c.E * (sizeof(float) + sizeof(int32_t));
  const size_t alone = aux_scratch_bytes(c);
  return fused > alone ? fused : alone;
}

void layout_of(const moe_config& c, moe_workspace_layout* L, size_t* total) {
  const size_t tk = static_cast<size_t>(c.T) * c.top_k;
  const size_t rows = static_cast<size_t>(max_rows_of(c));
  const size_t eb = elem_bytes(c.in_dtype);
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t at = off;
    off = align_up(off + bytes);
    return at;
  };
  L->scratch = take(dispatch_scratch_bytes(c));  // first, so moe_slice_dispatch can use the base
  L->expert_idx = take(tk * 4);
  L->gate_w = take(tk * 4);
  L->counts = take(static_cast<size_t>(c.local_count) * 4);
  L->offsets = take(static_cast<size_t>(c.local_count + 1) * 4);
  L->perm = take(rows * 4);
  L->inv_perm = take(tk * 4);
  L->x_sliced = take(rows * c.d * eb);
  L->H = take(rows * c.F * eb);
  L->y_sliced = take(rows * c.d * eb);
  L->gemm = take(grouped_gemm_workspace_bytes());
  L->logits = take(tk / c.top_k * c.E * 4);
  L->aux = take(aux_region_bytes(c));
  *total = off;
}

inline int hip_status(hipError_t e) { return e == hipSuccess ? MOE_OK : MOE_ERR_HIP; }

}  // namespace

extern "C" {

const char* moe_status_string(int status) {
  switch (status) {
    case MOE_OK: return "ok";
    case MOE_ERR_NULL: return "a required pointer is NULL";
    case MOE_ERR_SHAPE: return "a size is outside the supported range";
    case MOE_ERR_DTYPE: return "unsupported (in_dtype, out_dtype) pair";
    case MOE_ERR_ALIGN: return "a device pointer is not 16-byte aligned";
    case MOE_ERR_WORKSPACE: return "workspace too small";
    case MOE_ERR_HIP: return "a HIP runtime call failed";
    default: return "unknown status";
  }
}

int moe_init(void* stream) {
  void* scratch = nullptr;
  if (static_scratch_of_current_device(&scratch) != hipSuccess) return MOE_ERR_HIP;
  return hip_status(grouped_gemm_fast_init(static_cast<hipStream_t>(stream)));
}

int moe_set_option(int option, int64_t value) {
  if (value < 0 || value > 0x7fffffff) return MOE_ERR_SHAPE;
  switch (option) {
    case MOE_OPT_HANDOVER_DEVICE_SCOPE:
      grouped_gemm_fast_set_handover(value != 0, -1);
      return MOE_OK;
    case MOE_OPT_HANDOVER_SPIN_LIMIT:
      grouped_gemm_fast_set_handover(-1, static_cast<int>(value));
      return MOE_OK;
    default:
      return MOE_ERR_SHAPE;
  }
}

int64_t moe_capacity(const moe_config* cfg) {
  if (check_config(cfg) != MOE_OK) return -1;
  return capacity_of(*cfg);
}

int64_t moe_max_rows(const moe_config* cfg) {
  if (check_config(cfg) != MOE_OK) return 0;
  return max_rows_of(*cfg);
}

size_t moe_workspace_bytes(const moe_config* cfg) {
  if (check_config(cfg) != MOE_OK) return 0;
  moe_workspace_layout L;
  size_t total = 0;
  layout_of(*cfg, &L, &total);
  return total;
}

size_t moe_ffn_workspace_bytes(const moe_config* cfg) {
  if (check_config(cfg) != MOE_OK) return 0;
  return grouped_gemm_workspace_bytes();
}

size_t moe_dispatch_workspace_bytes(const moe_config* cfg) {
  if (check_config(cfg) != MOE_OK) return 0;
  return dispatch_scratch_bytes(*cfg);
}

int moe_workspace_offsets(const moe_config* cfg, moe_workspace_layout* layout) {
  int st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (layout == nullptr) return MOE_ERR_NULL;
  size_t total = 0;
  layout_of(*cfg, layout, &total);
  return MOE_OK;
}

int moe_gate(const moe_config* cfg, const void* x, const void* Wg, const float* bias,
             const float* logits_in, float* logits_out, int32_t* expert_idx, float* gate_w,
             void* stream) {
  int st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (expert_idx == nullptr || gate_w == nullptr) return MOE_ERR_NULL;
  if (logits_in == nullptr && (x == nullptr || Wg == nullptr)) return MOE_ERR_NULL;
  if (misaligned(x) || misaligned(Wg) || misaligned(bias) || misaligned(logits_in) ||
      misaligned(logits_out) || misaligned(expert_idx) || misaligned(gate_w))
    return MOE_ERR_ALIGN;
  return hip_status(launch_gate(*cfg, x, Wg, bias, logits_in, logits_out, expert_idx, gate_w,
                                static_cast<hipStream_t>(stream)));
}

size_t moe_aux_workspace_bytes(const moe_config* cfg) {
  if (check_config(cfg) != MOE_OK) return 0;
  return aux_scratch_bytes(*cfg);
}

int moe_aux_loss(const moe_config* cfg, const float* logits, const int32_t* expert_idx, float* l_aux,
                 float* mean_prob, int32_t* first_counts, void* workspace, size_t workspace_bytes,
                 void* stream) {
  int st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (l_aux == nullptr || workspace == nullptr) return MOE_ERR_NULL;
  if (cfg->T > 0 && (logits == nullptr || expert_idx == nullptr)) return MOE_ERR_NULL;
  if (misaligned(logits) || misaligned(expert_idx) || misaligned(mean_prob) ||
      misaligned(first_counts) || misaligned(workspace))
    return MOE_ERR_ALIGN;
  if (workspace_bytes < aux_scratch_bytes(*cfg)) return MOE_ERR_WORKSPACE;
  return hip_status(launch_aux_loss(*cfg, logits, expert_idx, l_aux, mean_prob, first_counts,
                                    workspace, static_cast<hipStream_t>(stream)));
}

int moe_slice_dispatch(const moe_config* cfg, const void* x, const int32_t* expert_idx,
                       int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                       void* x_sliced, void* workspace, size_t workspace_bytes, void* stream) {
  int st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (counts == nullptr || offsets == nullptr || workspace == nullptr) return MOE_ERR_NULL;
  if (cfg->T > 0 && (expert_idx == nullptr || perm == nullptr || inv_perm == nullptr))
    return MOE_ERR_NULL;  // with T == 0 the per-token arrays are empty and may be NULL
  if (cfg->T > 0 && x_sliced != nullptr && x == nullptr) return MOE_ERR_NULL;
  if (misaligned(x) || misaligned(expert_idx) || misaligned(counts) || misaligned(offsets) ||
      misaligned(perm) || misaligned(inv_perm) || misaligned(x_sliced) || misaligned(workspace))
    return MOE_ERR_ALIGN;
  if (workspace_bytes < dispatch_scratch_bytes(*cfg)) return MOE_ERR_WORKSPACE;
  hipStream_t s = static_cast<hipStream_t>(stream);
  hipError_t e = launch_permute(*cfg, capacity_of(*cfg), expert_idx, counts, offsets, perm, inv_perm,
                                static_cast<int32_t*>(workspace), s);
  if (e != hipSuccess) return MOE_ERR_HIP;
  if (x_sliced != nullptr)
    e = launch_slice(*cfg, x, perm, offsets, x_sliced, max_rows_of(*cfg), s);
  return hip_status(e);
}

static_assert(kStaticScratchBytes == MOE_STATIC_SCRATCH_BYTES, "header and library disagree");

int moe_slice_dispatch_static(const moe_config* cfg, const void* x, const int32_t* expert_idx,
                              int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                              void* x_sliced, void* stream) {
  int st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (dispatch_scratch_bytes(*cfg) > kStaticScratchBytes) return MOE_ERR_WORKSPACE;
  void* scratch = nullptr;
  if (static_scratch_of_current_device(&scratch) != hipSuccess) return MOE_ERR_HIP;
  return moe_slice_dispatch(cfg, x, expert_idx, counts, offsets, perm, inv_perm, x_sliced, scratch,
                            kStaticScratchBytes, stream);
}

int moe_slice_rows(const moe_config* cfg, const void* x, const int32_t* perm, const int32_t* offsets,
                   void* x_sliced, void* stream) {
  int st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (offsets == nullptr) return MOE_ERR_NULL;
  if (cfg->T > 0 && (x == nullptr || perm == nullptr || x_sliced == nullptr)) return MOE_ERR_NULL;
  if (misaligned(x) || misaligned(perm) || misaligned(offsets) || misaligned(x_sliced))
    return MOE_ERR_ALIGN;
  return hip_status(launch_slice(*cfg, x, perm, offsets, x_sliced, max_rows_of(*cfg),
                                 static_cast<hipStream_t>(stream)));
}

int moe_expert_ffn_up(const moe_config* cfg, const void* x_sliced, const int32_t* offsets,
                      const void* W1, void* H, void* workspace, size_t workspace_bytes,
                      void* stream) {
  int st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (x_sliced == nullptr || offsets == nullptr || W1 == nullptr || H == nullptr ||
      workspace == nullptr)
    return MOE_ERR_NULL;
  if (misaligned(x_sliced) || misaligned(offsets) || misaligned(W1) || misaligned(H) ||
      misaligned(workspace))
    return MOE_ERR_ALIGN;
  if (workspace_bytes < grouped_gemm_workspace_bytes()) return MOE_ERR_WORKSPACE;
  return hip_status(launch_grouped_gemm(cfg->in_dtype, true, x_sliced, W1, H, offsets,
                                        cfg->local_count, max_rows_of(*cfg), cfg->F, cfg->d,
                                        workspace, static_cast<hipStream_t>(stream)));
}

int moe_expert_ffn_down(const moe_config* cfg, const void* H, const int32_t* offsets,
                        const void* W2, void* y_sliced, void* workspace, size_t workspace_bytes,
                        void* stream) {
  int st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (H == nullptr || offsets == nullptr || W2 == nullptr || y_sliced == nullptr ||
      workspace == nullptr)
    return MOE_ERR_NULL;
  if (misaligned(H) || misaligned(offsets) || misaligned(W2) || misaligned(y_sliced) ||
      misaligned(workspace))
    return MOE_ERR_ALIGN;
  if (workspace_bytes < grouped_gemm_workspace_bytes()) return MOE_ERR_WORKSPACE;
  return hip_status(launch_grouped_gemm(cfg->in_dtype, false, H, W2, y_sliced, offsets,
                                        cfg->local_count, max_rows_of(*cfg), cfg->d, cfg->F,
                                        workspace, static_cast<hipStream_t>(stream)));
}

int moe_expert_ffn(const moe_config* cfg, const void* x_sliced, const int32_t* offsets,
                   const void* W1, const void* W2, void* H, void* y_sliced, void* workspace,
                   size_t workspace_bytes, void* stream) {
  if (W2 == nullptr || y_sliced == nullptr) return MOE_ERR_NULL;
  if (misaligned(W2) || misaligned(y_sliced)) return MOE_ERR_ALIGN;
  int st = moe_expert_ffn_up(cfg, x_sliced, offsets, W1, H, workspace, workspace_bytes, stream);
  if (st != MOE_OK) return st;
  return moe_expert_ffn_down(cfg, H, offsets, W2, y_sliced, workspace, workspace_bytes, stream);
}

size_t moe_ffn_backward_workspace_bytes(const moe_config* cfg) {
  if (check_config(cfg) != MOE_OK || !is_16bit(cfg->in_dtype)) return 0;
  return expert_ffn_backward_scratch_bytes(*cfg, max_rows_of(*cfg));
}

int moe_expert_ffn_backward(const moe_config* cfg, const void* x_sliced, const int32_t* offsets,
                            const void* W1, const void* W2, const void* dY, void* dX_sliced, float* dW1,
                            float* dW2, void* workspace, size_t workspace_bytes, void* stream) {
  int st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (!is_16bit(cfg->in_dtype)) return MOE_ERR_DTYPE;
  if (x_sliced == nullptr || offsets == nullptr || W1 == nullptr || W2 == nullptr || dY == nullptr ||
      dX_sliced == nullptr || dW1 == nullptr || dW2 == nullptr || workspace == nullptr)
    return MOE_ERR_NULL;
  if (misaligned(x_sliced) || misaligned(offsets) || misaligned(W1) || misaligned(W2) || misaligned(dY) ||
      misaligned(dX_sliced) || misaligned(dW1) || misaligned(dW2) || misaligned(workspace))
    return MOE_ERR_ALIGN;
  const int64_t rows = max_rows_of(*cfg);
  if (workspace_bytes < expert_ffn_backward_scratch_bytes(*cfg, rows)) return MOE_ERR_WORKSPACE;
  return hip_status(launch_expert_ffn_backward(*cfg, rows, x_sliced, offsets, W1, W2, dY, dX_sliced, dW1, dW2,
                                               workspace, static_cast<hipStream_t>(stream)));
}

namespace {

// Where moe_layer_backward keeps its intermediates.
struct backward_layout {
  size_t scratch, expert_idx, gate_w, counts, offsets, perm, inv_perm, logits, dlogits, row_dot, x_sliced, dY,
      dX_sliced, dwg, ffn;
};

void backward_layout_of(const moe_config& c, backward_layout* L, size_t* total) {
  const size_t tk = static_cast<size_t>(c.T) * c.top_k;
  const size_t rows = static_cast<size_t>(max_rows_of(c));
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t at = off;
    off = align_up(off + bytes);
    return at;
  };
  L->scratch = take(dispatch_scratch_bytes(c));
  L->expert_idx = take(tk * 4);
  L->gate_w = take(tk * 4);
  L->counts = take(static_cast<size_t>(c.local_count) * 4);
  L->offsets = take(static_cast<size_t>(c.local_count + 1) * 4);
  L->perm = take(rows * 4);
  L->inv_perm = take(tk * 4);
  L->logits = take(static_cast<size_t>(c.T) * c.E * 4);
  L->dlogits = take(static_cast<size_t>(c.T) * c.E * 4);
  L->row_dot = take(rows * 4);
  L->x_sliced = take(rows * c.d * 2);
  L->dY = take(rows * c.d * 2);
  L->dX_sliced = take(rows * c.d * 2);
  L->dwg = take(dwg_scratch_bytes(c));
  L->ffn = take(expert_ffn_backward_scratch_bytes(c, max_rows_of(c)));
  *total = off;
}

}  // namespace

size_t moe_layer_backward_workspace_bytes(const moe_config* cfg) {
  if (check_config(cfg) != MOE_OK || !is_16bit(cfg->in_dtype)) return 0;
  backward_layout L;
  size_t total = 0;
  backward_layout_of(*cfg, &L, &total);
  return total;
}

int moe_layer_backward(const moe_config* cfg, const void* x, const void* Wg, const float* bias, const void* W1,
                       const void* W2, const void* d_out, void* dx, float* dWg, float* dbias, float* dW1,
                       float* dW2, void* workspace, size_t workspace_bytes, void* stream) {
  int st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (!is_16bit(cfg->in_dtype)) return MOE_ERR_DTYPE;
  if (x == nullptr || Wg == nullptr || W1 == nullptr || W2 == nullptr || d_out == nullptr || dx == nullptr ||
      dWg == nullptr || dW1 == nullptr || dW2 == nullptr || workspace == nullptr)
    return MOE_ERR_NULL;
  if (misaligned(x) || misaligned(Wg) || misaligned(bias) || misaligned(W1) || misaligned(W2) ||
      misaligned(d_out) || misaligned(dx) || misaligned(dWg) || misaligned(dbias) || misaligned(dW1) ||
      misaligned(dW2) || misaligned(workspace))
    return MOE_ERR_ALIGN;
  backward_layout L;
  size_t total = 0;
  backward_layout_of(*cfg, &L, &total);
  if (workspace_bytes < total) return MOE_ERR_WORKSPACE;

  const moe_config& c = *cfg;
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  int32_t* expert_idx = reinterpret_cast<int32_t*>(ws + L.expert_idx);
  float* gate_w = reinterpret_cast<float*>(ws + L.gate_w);
  int32_t* counts = reinterpret_cast<int32_t*>(ws + L.counts);
  int32_t* offsets = reinterpret_cast<int32_t*>(ws + L.offsets);
  int32_t* perm = reinterpret_cast<int32_t*>(ws + L.perm);
  int32_t* inv_perm = reinterpret_cast<int32_t*>(ws + L.inv_perm);
  int32_t* seg_scratch = reinterpret_cast<int32_t*>(ws + L.scratch);
  float* logits = reinterpret_cast<float*>(ws + L.logits);
  float* dlogits = reinterpret_cast<float*>(ws + L.dlogits);
  float* row_dot = reinterpret_cast<float*>(ws + L.row_dot);
  const int64_t rows = max_rows_of(c);
#define PPMOE_TRY(expr)                            \
  do {                                             \
    if ((expr) != hipSuccess) return MOE_ERR_HIP;  \
  } while (0)
  // The forward's routing is recomputed (the gating kernel reads x once; nothing has to be kept from
  // the forward call), this time with the logits written out for the softmax's derivative.
  GateFusion fusion = {};
  const bool fused_gate = gate_is_fused_kernel(c);
  if (fused_gate) fusion.seg_count = seg_scratch;
  PPMOE_TRY(launch_gate(c, x, Wg, bias, nullptr, logits, expert_idx, gate_w, s, fused_gate ? &fusion : nullptr));
  if (fusion.seg_assign > 0)
    PPMOE_TRY(launch_permute(c, capacity_of(c), expert_idx, counts, offsets, perm, inv_perm, seg_scratch, s,
                             fusion.seg_assign, true, nullptr));
  else
    PPMOE_TRY(launch_permute(c, capacity_of(c), expert_idx, counts, offsets, perm, inv_perm, seg_scratch, s));
  PPMOE_TRY(launch_slice(c, x, perm, offsets, ws + L.x_sliced, rows, s));
  PPMOE_TRY(launch_gather_scale(c, d_out, perm, offsets, gate_w, ws + L.dY, rows, s));
  PPMOE_TRY(launch_expert_ffn_backward(c, rows, ws + L.x_sliced, offsets, W1, W2, ws + L.dY, ws + L.dX_sliced, dW1,
                                       dW2, ws + L.ffn, s, row_dot));
  PPMOE_TRY(launch_gate_backward(c, logits, expert_idx, gate_w, inv_perm, row_dot, dlogits, s));
  PPMOE_TRY(launch_dx(c, ws + L.dX_sliced, inv_perm, dlogits, Wg, dx, s));
  PPMOE_TRY(launch_dwg(c, x, dlogits, dWg, dbias, ws + L.dwg, s));
#undef PPMOE_TRY
  return MOE_OK;
}

static int layer_fuses(const moe_config& c);

namespace {

// What moe_layer_forward_train keeps for moe_layer_backward_saved.
struct saved_layout {
  size_t expert_idx, gate_w, offsets, perm, inv_perm, logits, x_sliced, U, H;
};

void saved_layout_of(const moe_config& c, saved_layout* L, size_t* total) {
  const size_t tk = static_cast<size_t>(c.T) * c.top_k;
  const size_t rows = static_cast<size_t>(max_rows_of(c));
  size_t off = 0;
  auto take = [&](size_t bytes) {
    size_t at = off;
    off = align_up(off + bytes);
    return at;
  };
  L->expert_idx = take(tk * 4);
  L->gate_w = take(tk * 4);
  L->offsets = take(static_cast<size_t>(c.local_count + 1) * 4);
  L->perm = take(rows * 4);
  L->inv_perm = take(tk * 4);
  L->logits = take(static_cast<size_t>(c.T) * c.E * 4);
  L->x_sliced = take(rows * c.d * 2);
  L->U = take(rows * c.F * 2);
  L->H = take(rows * c.F * 2);
  *total = off;
}

}  // namespace

size_t moe_layer_saved_bytes(const moe_config* cfg) {
  if (check_config(cfg) != MOE_OK || !is_16bit(cfg->in_dtype)) return 0;
  saved_layout S;
  size_t total = 0;
  saved_layout_of(*cfg, &S, &total);
  return total;
}

int moe_layer_forward_train(const moe_config* cfg, const void* x, const void* Wg, const float* bias,
                            const void* W1, const void* W2, void* out, float* l_aux, float* mean_prob,
                            int32_t* first_counts, void* saved, size_t saved_bytes, void* workspace,
                            size_t workspace_bytes, void* stream) {
  int st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (!is_16bit(cfg->in_dtype)) return MOE_ERR_DTYPE;
  if (x == nullptr || Wg == nullptr || W1 == nullptr || W2 == nullptr || out == nullptr || saved == nullptr ||
      workspace == nullptr)
    return MOE_ERR_NULL;
  if (l_aux == nullptr && (mean_prob != nullptr || first_counts != nullptr)) return MOE_ERR_NULL;
  if (misaligned(x) || misaligned(Wg) || misaligned(bias) || misaligned(W1) || misaligned(W2) ||
      misaligned(out) || misaligned(saved) || misaligned(workspace) || misaligned(mean_prob) ||
      misaligned(first_counts) || (reinterpret_cast<uintptr_t>(l_aux) & 3u) != 0)
    return MOE_ERR_ALIGN;
  moe_workspace_layout L;
  saved_layout S;
  size_t total = 0, saved_total = 0;
  layout_of(*cfg, &L, &total);
  saved_layout_of(*cfg, &S, &saved_total);
  if (workspace_bytes < total || saved_bytes < saved_total) return MOE_ERR_WORKSPACE;

  const moe_config& c = *cfg;
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  unsigned char* sv = static_cast<unsigned char*>(saved);
  int32_t* expert_idx = reinterpret_cast<int32_t*>(sv + S.expert_idx);
  float* gate_w = reinterpret_cast<float*>(sv + S.gate_w);
  int32_t* offsets = reinterpret_cast<int32_t*>(sv + S.offsets);
  int32_t* perm = reinterpret_cast<int32_t*>(sv + S.perm);
  int32_t* inv_perm = reinterpret_cast<int32_t*>(sv + S.inv_perm);
  float* logits = reinterpret_cast<float*>(sv + S.logits);
  void* x_sliced = sv + S.x_sliced;
  void* U = sv + S.U;
  void* H = sv + S.H;
  int32_t* counts = reinterpret_cast<int32_t*>(ws + L.counts);
  int32_t* seg_scratch = reinterpret_cast<int32_t*>(ws + L.scratch);
  void* y_sliced = ws + L.y_sliced;
  const int64_t rows = max_rows_of(c);
#define PPMOE_TRY(expr)                            \
  do {                                             \
    if ((expr) != hipSuccess) return MOE_ERR_HIP;  \
  } while (0)
  // Gating and permutation as in moe_layer_forward_aux, with the logits written out (the backward's
  // softmax derivative reads them).
  const bool want_aux = l_aux != nullptr;
  const bool fused_gate = gate_is_fused_kernel(c);
  GateFusion fusion = {};
  if (fused_gate) {
    fusion.seg_count = seg_scratch;
    if (want_aux) {
      fusion.part_prob = reinterpret_cast<float*>(ws + L.aux);
      fusion.part_cnt = reinterpret_cast<int32_t*>(fusion.part_prob + static_cast<size_t>(max_segments(c)) * c.E);
    }
  }
  PPMOE_TRY(launch_gate(c, x, Wg, bias, nullptr, logits, expert_idx, gate_w, s, fused_gate ? &fusion : nullptr));
  if (fusion.seg_assign > 0) {
    const AuxOut aux = {l_aux, mean_prob, first_counts, fusion.part_prob, fusion.part_cnt, fusion.n_seg, c.E, c.T};
    PPMOE_TRY(launch_permute(c, capacity_of(c), expert_idx, counts, offsets, perm, inv_perm, seg_scratch, s,
                             fusion.seg_assign, true, want_aux ? &aux : nullptr));
  } else {
    PPMOE_TRY(launch_permute(c, capacity_of(c), expert_idx, counts, offsets, perm, inv_perm, seg_scratch, s));
    if (want_aux)
      PPMOE_TRY(launch_aux_loss(c, logits, expert_idx, l_aux, mean_prob, first_counts, ws + L.aux, s));
  }
  // The sliced tokens and both sides of the activation stay for the backward: the first GEMM stores
  // U = X A, a pass over it H = GeLU(U).
  PPMOE_TRY(launch_slice(c, x, perm, offsets, x_sliced, rows, s));
  PPMOE_TRY(launch_grouped_gemm(c.in_dtype, false, x_sliced, W1, U, offsets, c.local_count, rows, c.F, c.d,
                                ws + L.gemm, s));
  PPMOE_TRY(launch_gelu_rows(c, U, H, offsets, rows, s));
  const int fuses = layer_fuses(c);
  if ((fuses & MOE_FUSE_COMBINE) && c.top_k == 1) {
    if (c.local_count < c.E || c.capacity_factor > 0.f)
      PPMOE_TRY(launch_zero_unrouted_rows(c, inv_perm, out, s));
    PPMOE_TRY(launch_grouped_gemm(c.in_dtype, false, H, W2, out, offsets, c.local_count, rows, c.d,
                                  c.F, ws + L.gemm, s, 2, perm, gate_w));
  } else if (fuses & MOE_FUSE_COMBINE) {
    PPMOE_TRY(launch_grouped_gemm(c.in_dtype, false, H, W2, out, offsets, c.local_count, rows, c.d,
                                  c.F, ws + L.gemm, s, 2, perm, gate_w, c.top_k, inv_perm, y_sliced));
    PPMOE_TRY(launch_combine(c, y_sliced, inv_perm, gate_w, out, s, true));
  } else {
    PPMOE_TRY(launch_grouped_gemm(c.in_dtype, false, H, W2, y_sliced, offsets, c.local_count, rows,
                                  c.d, c.F, ws + L.gemm, s));
    PPMOE_TRY(launch_combine(c, y_sliced, inv_perm, gate_w, out, s));
  }
#undef PPMOE_TRY
  return MOE_OK;
}

int moe_layer_backward_saved(const moe_config* cfg, const void* x, const void* Wg, const void* W1,
                             const void* W2, const void* d_out, const void* saved, size_t saved_bytes, void* dx,
                             float* dWg, float* dbias, float* dW1, float* dW2, void* workspace,
                             size_t workspace_bytes, void* stream) {
  int st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (!is_16bit(cfg->in_dtype)) return MOE_ERR_DTYPE;
  if (x == nullptr || Wg == nullptr || W1 == nullptr || W2 == nullptr || d_out == nullptr || saved == nullptr ||
      dx == nullptr || dWg == nullptr || dW1 == nullptr || dW2 == nullptr || workspace == nullptr)
    return MOE_ERR_NULL;
  if (misaligned(x) || misaligned(Wg) || misaligned(W1) || misaligned(W2) || misaligned(d_out) ||
      misaligned(saved) || misaligned(dx) || misaligned(dWg) || misaligned(dbias) || misaligned(dW1) ||
      misaligned(dW2) || misaligned(workspace))
    return MOE_ERR_ALIGN;
  backward_layout L;
  saved_layout S;
  size_t total = 0, saved_total = 0;
  backward_layout_of(*cfg, &L, &total);
  saved_layout_of(*cfg, &S, &saved_total);
  if (workspace_bytes < total || saved_bytes < saved_total) return MOE_ERR_WORKSPACE;

  const moe_config& c = *cfg;
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  const unsigned char* sv = static_cast<const unsigned char*>(saved);
  const int32_t* expert_idx = reinterpret_cast<const int32_t*>(sv + S.expert_idx);
  const float* gate_w = reinterpret_cast<const float*>(sv + S.gate_w);
  const int32_t* offsets = reinterpret_cast<const int32_t*>(sv + S.offsets);
  const int32_t* perm = reinterpret_cast<const int32_t*>(sv + S.perm);
  const int32_t* inv_perm = reinterpret_cast<const int32_t*>(sv + S.inv_perm);
  const float* logits = reinterpret_cast<const float*>(sv + S.logits);
  float* dlogits = reinterpret_cast<float*>(ws + L.dlogits);
  float* row_dot = reinterpret_cast<float*>(ws + L.row_dot);
  const int64_t rows = max_rows_of(c);
#define PPMOE_TRY(expr)                            \
  do {                                             \
    if ((expr) != hipSuccess) return MOE_ERR_HIP;  \
  } while (0)
  PPMOE_TRY(launch_gather_scale(c, d_out, perm, offsets, gate_w, ws + L.dY, rows, s));
  PPMOE_TRY(launch_expert_ffn_backward(c, rows, sv + S.x_sliced, offsets, W1, W2, ws + L.dY, ws + L.dX_sliced, dW1,
                                       dW2, ws + L.ffn, s, row_dot, sv + S.U, sv + S.H));
  PPMOE_TRY(launch_gate_backward(c, logits, expert_idx, gate_w, inv_perm, row_dot, dlogits, s));
  PPMOE_TRY(launch_dx(c, ws + L.dX_sliced, inv_perm, dlogits, Wg, dx, s));
  PPMOE_TRY(launch_dwg(c, x, dlogits, dWg, dbias, ws + L.dwg, s));
#undef PPMOE_TRY
  return MOE_OK;
}

int moe_ffn_check(const moe_config* cfg, const void* workspace, int layer_workspace,
                  int32_t* status, void* stream) {
  int st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (workspace == nullptr || status == nullptr) return MOE_ERR_NULL;
  const unsigned char* ws = static_cast<const unsigned char*>(workspace);
  if (layer_workspace) {
    moe_workspace_layout L;
    size_t total = 0;
    layout_of(*cfg, &L, &total);
    ws += L.gemm;
  }
  uint32_t word = 0;
  if (read_gemm_error_word(ws, &word, static_cast<hipStream_t>(stream)) != hipSuccess)
    return MOE_ERR_HIP;
  *status = (word & 0xffffff00u) == kGemmErrorMagic ? static_cast<int32_t>(word & 0xffu) : 0;
  return MOE_OK;
}

int moe_ffn_clock(const moe_config* cfg, const void* workspace, int layer_workspace, double* shader_ghz,
                  double* kernel_us, void* stream) {
  int st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (workspace == nullptr || shader_ghz == nullptr || kernel_us == nullptr) return MOE_ERR_NULL;
  const unsigned char* ws = static_cast<const unsigned char*>(workspace);
  if (layer_workspace) {
    moe_workspace_layout L;
    size_t total = 0;
    layout_of(*cfg, &L, &total);
    ws += L.gemm;
  }
  uint64_t shader = 0, wall = 0;
  if (read_gemm_clock_words(ws, &shader, &wall, static_cast<hipStream_t>(stream)) != hipSuccess)
    return MOE_ERR_HIP;
  int dev = 0, wall_khz = 0;
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&wall_khz, hipDeviceAttributeWallClockRate, dev) != hipSuccess || wall_khz <= 0)
    return MOE_ERR_HIP;
  if (wall == 0 || wall > (1ull << 40) || shader > (1ull << 50)) {   // (no fast-path launch has written the words)
    *shader_ghz = 0.0;
    *kernel_us = 0.0;
    return MOE_OK;
  }
  *kernel_us = static_cast<double>(wall) / wall_khz * 1e3;
  *shader_ghz = static_cast<double>(shader) / static_cast<double>(wall) * wall_khz * 1e-6;
  return MOE_OK;
}

int moe_combine(const moe_config* cfg, const void* y_sliced, const int32_t* inv_perm,
                const float* gate_w, void* out, void* stream) {
  int st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (y_sliced == nullptr || inv_perm == nullptr || gate_w == nullptr || out == nullptr)
    return MOE_ERR_NULL;
  if (misaligned(y_sliced) || misaligned(inv_perm) || misaligned(gate_w) || misaligned(out))
    return MOE_ERR_ALIGN;
  return hip_status(launch_combine(*cfg, y_sliced, inv_perm, gate_w, out,
                                   static_cast<hipStream_t>(stream)));
}

// What moe_layer_forward folds into the expert GEMMs on the 16-bit fast path.  Bit 0: the first GEMM
// reads the token rows through the permutation, so the sliced copy of the tokens is not made.
// Bit 1 (output of the input type): the second GEMM multiplies by the gate weight and stores straight
// into the layer output every row that is its token's only kept local pick (all of them under top-1:
// the packed expert outputs are then not made at all; under top-k the others still go through
// y_sliced and the combine kernel, which leaves the placed rows alone).
static int layer_fuses(const moe_config& c) {
  if (!grouped_gemm_can_fuse(c.in_dtype, c.d, c.T)) return 0;
  int f = MOE_FUSE_SLICE;
  if (c.out_dtype == c.in_dtype && grouped_gemm_is_fast(c.in_dtype, c.F)) f |= MOE_FUSE_COMBINE;
  return f;
}

int moe_layer_fuses(const moe_config* cfg) {
  if (check_config(cfg) != MOE_OK) return 0;
  return layer_fuses(*cfg);
}

int moe_layer_forward_aux(const moe_config* cfg, const void* x, const void* Wg, const float* bias,
                          const void* W1, const void* W2, void* out, float* l_aux, float* mean_prob,
                          int32_t* first_counts, void* workspace, size_t workspace_bytes,
                          void* const* stage_events, void* stream) {
  int st = check_config(cfg);
  if (st != MOE_OK) return st;
  if (x == nullptr || Wg == nullptr || W1 == nullptr || W2 == nullptr || out == nullptr ||
      workspace == nullptr)
    return MOE_ERR_NULL;
  if (l_aux == nullptr && (mean_prob != nullptr || first_counts != nullptr)) return MOE_ERR_NULL;
  if (misaligned(x) || misaligned(Wg) || misaligned(bias) || misaligned(W1) || misaligned(W2) ||
      misaligned(out) || misaligned(workspace) || misaligned(mean_prob) || misaligned(first_counts) ||
      (reinterpret_cast<uintptr_t>(l_aux) & 3u) != 0)
    return MOE_ERR_ALIGN;
  moe_workspace_layout L;
  size_t total = 0;
  layout_of(*cfg, &L, &total);
  if (workspace_bytes < total) return MOE_ERR_WORKSPACE;
  if (stage_events != nullptr)
    for (int i = 0; i <= MOE_NUM_STAGES; ++i)
      if (stage_events[i] == nullptr) return MOE_ERR_NULL;

  const moe_config& c = *cfg;
  hipStream_t s = static_cast<hipStream_t>(stream);
  unsigned char* ws = static_cast<unsigned char*>(workspace);
  int32_t* expert_idx = reinterpret_cast<int32_t*>(ws + L.expert_idx);
  float* gate_w = reinterpret_cast<float*>(ws + L.gate_w);
  int32_t* counts = reinterpret_cast<int32_t*>(ws + L.counts);
  int32_t* offsets = reinterpret_cast<int32_t*>(ws + L.offsets);
  int32_t* perm = reinterpret_cast<int32_t*>(ws + L.perm);
  int32_t* inv_perm = reinterpret_cast<int32_t*>(ws + L.inv_perm);
  int32_t* seg_scratch = reinterpret_cast<int32_t*>(ws + L.scratch);
  float* logits = reinterpret_cast<float*>(ws + L.logits);
  void* x_sliced = ws + L.x_sliced;
  void* H = ws + L.H;
  void* y_sliced = ws + L.y_sliced;
  const int64_t rows = max_rows_of(c);

  auto mark = [&](int i) -> hipError_t {
    if (stage_events == nullptr) return hipSuccess;
    return hipEventRecord(static_cast<hipEvent_t>(stage_events[i]), s);
  };
  hipError_t e;
#define PPMOE_TRY(expr)                  \
  do {                                   \
    e = (expr);                          \
    if (e != hipSuccess) return MOE_ERR_HIP; \
  } while (0)

  // Gating.  Where the router runs in the kernel that holds Wg in LDS, that kernel also counts the
  // picks per segment of the permutation (one launch less below) and, when the balance loss is
  // wanted, leaves its partial sums; the permutation's scan launch then finishes the loss.
  const bool want_aux = l_aux != nullptr;
  const bool fused_gate = gate_is_fused_kernel(c);
  GateFusion fusion = {};
  if (fused_gate) {
    fusion.seg_count = seg_scratch;
    if (want_aux) {
      fusion.part_prob = reinterpret_cast<float*>(ws + L.aux);
      fusion.part_cnt = reinterpret_cast<int32_t*>(fusion.part_prob + static_cast<size_t>(max_segments(c)) * c.E);
    }
  }
  PPMOE_TRY(mark(MOE_STAGE_GATE));
  PPMOE_TRY(launch_gate(c, x, Wg, bias, nullptr, (want_aux && !fused_gate) ? logits : nullptr, expert_idx,
                        gate_w, s, fused_gate ? &fusion : nullptr));
  PPMOE_TRY(mark(MOE_STAGE_PERMUTE));
  if (fusion.seg_assign > 0) {
    const AuxOut aux = {l_aux, mean_prob, first_counts, fusion.part_prob, fusion.part_cnt, fusion.n_seg, c.E, c.T};
    PPMOE_TRY(launch_permute(c, capacity_of(c), expert_idx, counts, offsets, perm, inv_perm, seg_scratch, s,
                             fusion.seg_assign, true, want_aux ? &aux : nullptr));
  } else {
    PPMOE_TRY(launch_permute(c, capacity_of(c), expert_idx, counts, offsets, perm, inv_perm, seg_scratch, s));
    if (want_aux)
      PPMOE_TRY(launch_aux_loss(c, logits, expert_idx, l_aux, mean_prob, first_counts, ws + L.aux, s));
  }
  // (a stage folded into a GEMM is empty; its events are still recorded)
  const int fuses = layer_fuses(c);
  PPMOE_TRY(mark(MOE_STAGE_SLICE));
  if (!(fuses & MOE_FUSE_SLICE)) PPMOE_TRY(launch_slice(c, x, perm, offsets, x_sliced, rows, s));
  PPMOE_TRY(mark(MOE_STAGE_FFN_UP));
  if (fuses & MOE_FUSE_SLICE)
    PPMOE_TRY(launch_grouped_gemm(c.in_dtype, true, x, W1, H, offsets, c.local_count, rows, c.F, c.d,
                                  ws + L.gemm, s, 1, perm, nullptr, c.top_k));
  else
    PPMOE_TRY(launch_grouped_gemm(c.in_dtype, true, x_sliced, W1, H, offsets, c.local_count, rows,
                                  c.F, c.d, ws + L.gemm, s));
  PPMOE_TRY(mark(MOE_STAGE_FFN_DOWN));
  if ((fuses & MOE_FUSE_COMBINE) && c.top_k == 1) {
    // Tokens without a kept local pick exist only with a subset of the experts or a capacity limit.
    if (c.local_count < c.E || c.capacity_factor > 0.f)
      PPMOE_TRY(launch_zero_unrouted_rows(c, inv_perm, out, s));
    PPMOE_TRY(launch_grouped_gemm(c.in_dtype, false, H, W2, out, offsets, c.local_count, rows, c.d,
                                  c.F, ws + L.gemm, s, 2, perm, gate_w));
    PPMOE_TRY(mark(MOE_STAGE_COMBINE));
  } else if (fuses & MOE_FUSE_COMBINE) {
    // top-k: rows that are their token's only kept local pick go straight into `out`; the combine
    // kernel then writes the other tokens (sums of several picks, and zero rows) and skips those.
    PPMOE_TRY(launch_grouped_gemm(c.in_dtype, false, H, W2, out, offsets, c.local_count, rows, c.d,
                                  c.F, ws + L.gemm, s, 2, perm, gate_w, c.top_k, inv_perm, y_sliced));
    PPMOE_TRY(mark(MOE_STAGE_COMBINE));
    PPMOE_TRY(launch_combine(c, y_sliced, inv_perm, gate_w, out, s, true));
  } else {
    PPMOE_TRY(launch_grouped_gemm(c.in_dtype, false, H, W2, y_sliced, offsets, c.local_count, rows,
                                  c.d, c.F, ws + L.gemm, s));
    PPMOE_TRY(mark(MOE_STAGE_COMBINE));
    PPMOE_TRY(launch_combine(c, y_sliced, inv_perm, gate_w, out, s));
  }
  PPMOE_TRY(mark(MOE_NUM_STAGES));
#undef PPMOE_TRY
  return MOE_OK;
}

int moe_layer_forward(const moe_config* cfg, const void* x, const void* Wg, const float* bias,
                      const void* W1, const void* W2, void* out, void* workspace,
                      size_t workspace_bytes, void* const* stage_events, void* stream) {
  return moe_layer_forward_aux(cfg, x, Wg, bias, W1, W2, out, nullptr, nullptr, nullptr, workspace,
                               workspace_bytes, stage_events, stream);
}

int moe_copy_bytes(const void* src, void* dst, size_t bytes, void* stream) {
  if (src == nullptr || dst == nullptr) return MOE_ERR_NULL;
  if (misaligned(src) || misaligned(dst)) return MOE_ERR_ALIGN;
  if (bytes % 16 != 0) return MOE_ERR_SHAPE;
  return hip_status(launch_copy_bytes(src, dst, static_cast<int64_t>(bytes),
                                      static_cast<hipStream_t>(stream)));
}

int moe_mfma_probe(int64_t iters, int random_operands, float* sink, double* flops, void* stream) {
  if (sink == nullptr || flops == nullptr) return MOE_ERR_NULL;
  if (iters < 0) return MOE_ERR_SHAPE;
  int blocks = 0;
  const hipError_t e = launch_mfma_probe(iters, random_operands, sink, &blocks,
                                         static_cast<hipStream_t>(stream));
  // per block: 4 wavefronts x 16 MFMAs of 2*32*32*16 flop per iteration
  *flops = static_cast<double>(blocks) * 4.0 * 16.0 * 32768.0 * static_cast<double>(iters);
  return hip_status(e);
}

int moe_event_create(void** event) {
  if (event == nullptr) return MOE_ERR_NULL;
  hipEvent_t ev;
  if (hipEventCreate(&ev) != hipSuccess) return MOE_ERR_HIP;
  *event = ev;
  return MOE_OK;
}

int moe_event_destroy(void* event) {
  if (event == nullptr) return MOE_ERR_NULL;
  return hip_status(hipEventDestroy(static_cast<hipEvent_t>(event)));
}

int moe_event_record(void* event, void* stream) {
  if (event == nullptr) return MOE_ERR_NULL;
  return hip_status(hipEventRecord(static_cast<hipEvent_t>(event), static_cast<hipStream_t>(stream)));
}

int moe_event_elapsed_ms(void* start, void* stop, float* ms) {
  if (start == nullptr || stop == nullptr || ms == nullptr) return MOE_ERR_NULL;
  if (hipEventSynchronize(static_cast<hipEvent_t>(stop)) != hipSuccess) return MOE_ERR_HIP;
  return hip_status(hipEventElapsedTime(ms, static_cast<hipEvent_t>(start),
                                        static_cast<hipEvent_t>(stop)));
}

}  // extern "C"
