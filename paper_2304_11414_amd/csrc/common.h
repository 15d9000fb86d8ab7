// Internal declarations shared by the kernels of libppmoe.so (gfx950 only).
#pragma once

#include <hip/hip_runtime.h>
#include <stdint.h>

#include <atomic>

#include "ppmoe.h"

namespace ppmoe {

constexpr int kWave = 64;          // CDNA wavefront
constexpr int kMaxExperts = 256;   // E limit of the ABI
constexpr int kMaxTopK = 8;
constexpr int kSegment = 64;       // assignments per segment of the permutation when it counts them itself
constexpr int kGateTokens = 16;    // tokens one wavefront of the bf16 gating kernel scores at a time

typedef uint16_t bf16_t;           // raw bf16 bits in memory
typedef uint32_t u32x4 __attribute__((ext_vector_type(4)));  // one 16-byte piece
typedef float f32x4 __attribute__((ext_vector_type(4)));

__device__ __forceinline__ float bf16_to_f32(bf16_t b) {
  return __uint_as_float(static_cast<uint32_t>(b) << 16);
}

// Round to nearest even; NaN stays a quiet NaN.
__device__ __forceinline__ bf16_t f32_to_bf16(float f) {
  uint32_t u = __float_as_uint(f);
  if ((u & 0x7fffffffu) > 0x7f800000u) return static_cast<bf16_t>((u >> 16) | 0x40u);
  u += 0x7fffu + ((u >> 16) & 1u);
  return static_cast<bf16_t>(u >> 16);
}

// Two floats -> two bf16 in one 32-bit word (lo in bits 0..15), round to nearest even: the
// hardware's packed conversion (v_cvt_pk_bf16_f32).
typedef __bf16 bf16x2_t __attribute__((ext_vector_type(2)));
typedef float f32x2_t __attribute__((ext_vector_type(2)));
__device__ __forceinline__ uint32_t pack_bf16x2(float lo, float hi) {
  f32x2_t v = {lo, hi};
  return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, bf16x2_t));
}

// Where the balance loss (Algorithm 1's l_aux) goes, and the per-segment partial sums it is made of:
// part_prob / part_cnt [n_part, E] (sum of the softmax probabilities and number of first picks per
// expert over the tokens of a segment).  l_aux == nullptr: no loss wanted.
struct AuxOut {
  float* l_aux;
  float* mean_prob;        // [E] or nullptr
  int32_t* first_counts;   // [E] or nullptr
  const float* part_prob;
  const int32_t* part_cnt;
  int n_part, E, T;
};

// What the fused gating kernel can do on the way (launch_gate, bf16 only): count the picks per
// permutation segment, and leave the partial sums of the balance loss.
struct GateFusion {
  int32_t* seg_count;   // [local_count, n_seg] or nullptr
  float* part_prob;     // [n_seg, E] or nullptr
  int32_t* part_cnt;    // [n_seg, E] or nullptr
  int seg_assign;       // out: assignments per segment the kernel used (0: it did not take this path)
  int n_seg;            // out
};

// The two 16-bit element types (MOE_BF16, MOE_F16; the paper trains in fp16, Section 4.1): what the
// matrix instructions and the conversions look like for each.  Both are raw 16-bit words in memory.
typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(8 * sizeof(_Float16)))) _Float16 f16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;
typedef _Float16 f16x2_t __attribute__((ext_vector_type(2)));

template <int DT>
struct Elem16;
template <>
struct Elem16<MOE_BF16> {
  typedef bf16x8 vec8;
  static __device__ __forceinline__ f32x16 mfma32(vec8 a, vec8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ f32x4 mfma16(vec8 a, vec8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_bf16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) { return pack_bf16x2(lo, hi); }
  static __device__ __forceinline__ float widen(uint16_t b) { return bf16_to_f32(b); }
  // the two halves of a 32-bit word holding two elements (lo in bits 0..15)
  static __device__ __forceinline__ void widen2(uint32_t w, float& lo, float& hi) {
    lo = __uint_as_float(w << 16);
    hi = __uint_as_float(w & 0xffff0000u);
  }
};
template <>
struct Elem16<MOE_F16> {
  typedef f16x8 vec8;
  static __device__ __forceinline__ f32x16 mfma32(vec8 a, vec8 b, f32x16 c) {
    return __builtin_amdgcn_mfma_f32_32x32x16_f16(a, b, c, 0, 0, 0);
  }
  static __device__ __forceinline__ f32x4 mfma16(vec8 a, vec8 b, f32x4 c) {
    return __builtin_amdgcn_mfma_f32_16x16x32_f16(a, b, c, 0, 0, 0);
  }
  // round to nearest even (the default rounding mode of the conversion)
  static __device__ __forceinline__ uint32_t pack2(float lo, float hi) {
    f32x2_t v = {lo, hi};
    return __builtin_bit_cast(uint32_t, __builtin_convertvector(v, f16x2_t));
  }
  static __device__ __forceinline__ float widen(uint16_t b) {
    return static_cast<float>(__builtin_bit_cast(_Float16, b));
  }
  static __device__ __forceinline__ void widen2(uint32_t w, float& lo, float& hi) {
    const f16x2_t v = __builtin_bit_cast(f16x2_t, w);
    lo = static_cast<float>(v.x);
    hi = static_cast<float>(v.y);
  }
};
inline bool is_16bit(int dtype) { return dtype == MOE_BF16 || dtype == MOE_F16; }

// Launchers (host).  Each returns the hipError_t of its last launch.
hipError_t launch_gate(const moe_config& c, const void* x, const void* Wg, const float* bias,
                       const float* logits_in, float* logits_out, int32_t* expert_idx,
                       float* gate_w, hipStream_t s, GateFusion* fusion = nullptr);
// Does launch_gate take the kernel that can honour a GateFusion request for this configuration?
bool gate_is_fused_kernel(const moe_config& c);

// seg_scratch: int32[local_count * max_segments * 2 + local_count] device scratch.
// seg_assign: consecutive assignments per segment; counted: seg_scratch already holds the
// per-segment counts (written by the gating kernel); aux: see AuxOut (may be nullptr).
hipError_t launch_permute(const moe_config& c, int64_t cap, const int32_t* expert_idx,
                          int32_t* counts, int32_t* offsets, int32_t* perm, int32_t* inv_perm,
                          int32_t* seg_scratch, hipStream_t s, int seg_assign = kSegment,
                          bool counted = false, const AuxOut* aux = nullptr);

// Runs `set_up` (returning hipError_t) the first time it is reached with a given device current and
// remembers, per device, that it has run: kernel attributes such as the dynamic-LDS limit belong to
// the device they were set on.  `done`: one bit per device ordinal (devices beyond 63 run it every
// time; the attributes are idempotent, as is a race between two first calls).
template <typename F>
inline hipError_t once_per_device(std::atomic<uint64_t>& done, F set_up) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  const uint64_t bit = dev >= 0 && dev < 64 ? uint64_t(1) << dev : 0;
  if (bit != 0 && (done.load(std::memory_order_acquire) & bit)) return hipSuccess;
  e = set_up();
  if (e == hipSuccess && bit != 0) done.fetch_or(bit, std::memory_order_release);
  return e;
}

// Allocation-free dispatch: device address of this device's file-scope scratch array of
// kStaticScratchBytes bytes (looked up on the first call per device, with that device current).
constexpr size_t kStaticScratchBytes = 4u << 20;
hipError_t static_scratch_of_current_device(void** ptr);

hipError_t launch_slice(const moe_config& c, const void* x, const int32_t* perm,
                        const int32_t* offsets, void* x_sliced, int64_t max_rows, hipStream_t s);

// skip_single: rows of tokens with exactly one kept local pick are left alone (the second GEMM has
// already placed them, see launch_grouped_gemm fuse 2).
hipError_t launch_combine(const moe_config& c, const void* y_sliced, const int32_t* inv_perm,
                          const float* gate_w, void* out, hipStream_t s, bool skip_single = false);

// Auxiliary balance loss from the logits and the picks; scratch: aux_scratch_bytes(c) bytes.
size_t aux_scratch_bytes(const moe_config& c);
hipError_t launch_aux_loss(const moe_config& c, const float* logits, const int32_t* expert_idx,
                           float* l_aux, float* mean_prob, int32_t* first_counts, void* scratch,
                           hipStream_t s);
// out[t, :] = +0 for every token t with inv_perm[t] < 0 (top-1 layout of inv_perm).
hipError_t launch_zero_unrouted_rows(const moe_config& c, const int32_t* inv_perm, void* out,
                                     hipStream_t s);
hipError_t launch_copy_bytes(const void* src, void* dst, int64_t bytes, hipStream_t s);
// Register-resident MFMA loop on one block per CU (at most kMaxPersistentBlocks); sink: one float per thread.
hipError_t launch_mfma_probe(int64_t iters, int random_operands, float* sink, int* blocks_out,
                             hipStream_t s);

// C[r, :] = act(A[r, :] . B[i]^T) for offsets[i] <= r < offsets[i+1];  A [rows, K], B [n_exp, Nout, K].
// workspace: grouped_gemm_workspace_bytes() of device scratch (partial sums of tiles cut between CUs).
// fuse (only where grouped_gemm_can_fuse says so): 1: packed row r of A is row aux_rows[r] / aux_div
// of the matrix given as A (first GEMM); 2 (second GEMM): packed row r of the result belongs to
// assignment a = aux_rows[r] of token a / aux_div; if it is the only entry >= 0 of aux_inv[token, :]
// it is stored, times aux_w[a], as row `token` of C (written by nobody else); else unweighted as
// packed row r of C2 (aux_div == 1: always the former, aux_inv and C2 are not used).
hipError_t launch_grouped_gemm(int in_dtype, bool gelu, const void* A, const void* B, void* C,
                               const int32_t* offsets, int n_exp, int64_t max_rows, int Nout, int K,
                               void* workspace, hipStream_t s, int fuse = 0,
                               const int32_t* aux_rows = nullptr, const float* aux_w = nullptr,
                               int aux_div = 1, const int32_t* aux_inv = nullptr, void* C2 = nullptr);
// Backward of the expert FFN on the packed rows (16-bit types only): dX [rows, d] 16-bit,
// dW1 [n_exp, F, d] and dW2 [n_exp, d, F] float32; scratch: expert_ffn_backward_scratch_bytes bytes.
size_t expert_ffn_backward_scratch_bytes(const moe_config& c, int64_t rows);
hipError_t launch_expert_ffn_backward(const moe_config& c, int64_t rows, const void* x_sliced,
                                      const int32_t* offsets, const void* W1, const void* W2,
                                      const void* dY, void* dX, float* dW1, float* dW2, void* scratch,
                                      hipStream_t s, float* row_dot = nullptr, const void* U_saved = nullptr,
                                      const void* H_saved = nullptr);
// U_saved, H_saved (both or neither): the pre-activations U = X A and H = GeLU(U) [rows, F] kept by a
// forward call; then U is not recomputed and H is not written.
// H = GeLU(U) over the packed rows [0, offsets[n_exp]) x F (16-bit types), the arithmetic of the
// backward's activation kernel.
hipError_t launch_gelu_rows(const moe_config& c, const void* U, void* H, const int32_t* offsets, int64_t rows,
                            hipStream_t s);
// row_dot (may be nullptr): [rows] float32, row_dot[r] = <dY[r, :], y_sliced[r, :]> (the derivative
// with respect to a scale factor of row r of the expert output).

// The pieces of the layer's backward that are not the expert FFN (layer_bwd.hip).
// dY[r, :] = gate_w[perm[r]] * d_out[perm[r] / k, :]  (d_out in out_dtype, dY in in_dtype)
hipError_t launch_gather_scale(const moe_config& c, const void* d_out, const int32_t* perm,
                               const int32_t* offsets, const float* gate_w, void* dY, int64_t max_rows,
                               hipStream_t s);
// dlogits[t, :] from the logits, the picks, the gate weights and row_dot (see gate backward in the header)
hipError_t launch_gate_backward(const moe_config& c, const float* logits, const int32_t* expert_idx,
                                const float* gate_w, const int32_t* inv_perm, const float* row_dot,
                                float* dlogits, hipStream_t s);
// dx[t, :] = sum over kept local picks of dX_sliced[inv_perm[t, j], :] + dlogits[t, :] Wg   (in_dtype)
hipError_t launch_dx(const moe_config& c, const void* dX_sliced, const int32_t* inv_perm,
                     const float* dlogits, const void* Wg, void* dx, hipStream_t s);
// dWg[e, :] = sum_t dlogits[t, e] x[t, :],  dbias[e] = sum_t dlogits[t, e]; scratch: dwg_scratch_bytes(c)
size_t dwg_scratch_bytes(const moe_config& c);
hipError_t launch_dwg(const moe_config& c, const void* x, const float* dlogits, float* dWg, float* dbias,
                      void* scratch, hipStream_t s);

inline bool grouped_gemm_is_fast(int in_dtype, int K) {
  return is_16bit(in_dtype) && (K % 64) == 0 && K < (1 << 22);   // 32-bit panel offsets in the fast kernel
}
// Can A be read through a row list?  Its byte offsets must fit the 32-bit offsets of the loads.
inline bool grouped_gemm_can_fuse(int in_dtype, int K, int64_t a_rows) {
  return grouped_gemm_is_fast(in_dtype, K) && a_rows * K * 2 < 0x7fffffffLL;
}

// bf16 fast path of the above (K a multiple of 64): persistent, at most kMaxPersistentBlocks blocks.
constexpr int kMaxPersistentBlocks = 256;
size_t grouped_gemm_fast_workspace_bytes();
// The fast GEMM leaves kGemmErrorMagic | code in one word of its workspace when a hand-over of
// partial sums did not take place (1: a partial sum did not arrive within the spin limit, 2: writer
// and reader were not on the same XCD although the set-up check said they would be); the reading
// CU then computed the missing part of the tile itself, so the output is complete either way.
constexpr uint32_t kGemmErrorMagic = 0x4d6f4500u;
// Copies that word to the host and synchronises the stream.
hipError_t read_gemm_error_word(const void* workspace, uint32_t* word, hipStream_t s);
hipError_t read_gemm_clock_words(const void* workspace, uint64_t* shader_ticks, uint64_t* wall_ticks,
                                 hipStream_t s);
inline size_t grouped_gemm_workspace_bytes() { return grouped_gemm_fast_workspace_bytes(); }
// Per-device set-up of the fast GEMM (kernel attributes, placement check); synchronises `s` once.
hipError_t grouped_gemm_fast_init(hipStream_t s);
// Diagnostic switches of the hand-over; a negative value leaves a setting as it is.
// force_device_scope: 1 = every hand-over uses device-scope fences whatever the placement check said.
// spin_limit: polls of a flag before the reader gives up and computes the missing k range itself
// (0 = never wait).
void grouped_gemm_fast_set_handover(int force_device_scope, int spin_limit);
hipError_t launch_grouped_gemm_fast(int in_dtype, bool gelu, const bf16_t* A, const bf16_t* B, bf16_t* C,
                                    const int32_t* offsets, int n_exp, int64_t max_rows, int Nout,
                                    int K, void* workspace, hipStream_t s, int fuse,
                                    const int32_t* aux_rows, const float* aux_w, int aux_div,
                                    const int32_t* aux_inv, bf16_t* C2);

// Most segments the permutation can be asked for: kSegment assignments each when it counts them
// itself, the tokens of one wavefront of the gating kernel each when that kernel counts them.
inline int64_t max_segments(const moe_config& c) {
  const int64_t a = static_cast<int64_t>(c.T) * c.top_k;
  const int64_t by_assign = (a + kSegment - 1) / kSegment;
  const int64_t by_tokens = (static_cast<int64_t>(c.T) + kGateTokens - 1) / kGateTokens;
  return by_assign > by_tokens ? by_assign : by_tokens;
}

}  // namespace ppmoe
