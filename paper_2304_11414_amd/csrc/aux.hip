// Auxiliary load-balance loss, the second value Algorithm 1 returns ("l_aux").  The paper takes it
// from GShard (Section 4.1) and prints no formula; this is the GShard form:
//
//   l_aux = E * sum_e mean_prob[e] * first_count[e] / T
//
// mean_prob[e] = mean over the tokens of softmax(logits)[t, e]; first_count[e] = number of tokens
// whose first pick is expert e (under top-2 gating too, before any capacity drop).
//
// Two launches: every wavefront reduces 64 tokens (probabilities by a fixed-order butterfly, first
// picks by ballot/popcount) and writes one partial sum per expert; one block then adds the partial
// sums in wavefront order.  No atomics: the float32 sums have a fixed order and the result is
// bitwise reproducible.

#include "common.h"

namespace ppmoe {

__global__ __launch_bounds__(256) void aux_partial_kernel(const float* __restrict__ logits,
                                                          const int32_t* __restrict__ expert_idx,
                                                          float* __restrict__ part_prob,
                                                          int32_t* __restrict__ part_cnt, int T,
                                                          int E, int k) {
  const int lane = threadIdx.x & 63;
  const int wave = blockIdx.x * 4 + (threadIdx.x >> 6);
  const int t = wave * kWave + lane;
  if (wave * kWave >= T) return;   // the whole wavefront is past the end
  const bool valid = t < T;
  const float* lg = logits + static_cast<size_t>(valid ? t : T - 1) * E;
  // the softmax of one token, as in the gating module: max-subtracted, float32
  float m = lg[0];
  for (int e = 1; e < E; ++e) m = fmaxf(m, lg[e]);
  float sum = 0.f;
  for (int e = 0; e < E; ++e) sum += expf(lg[e] - m);
  const int first = valid ? expert_idx[static_cast<size_t>(t) * k] : -1;
  for (int e = 0; e < E; ++e) {
    float p = valid ? expf(lg[e] - m) / sum : 0.f;
#pragma unroll
    for (int off = 32; off >= 1; off >>= 1) p += __shfl_xor(p, off, 64);
    const int cnt = __popcll(__ballot(first == e));
    if (lane == 0) {
      part_prob[static_cast<size_t>(wave) * E + e] = p;
      part_cnt[static_cast<size_t>(wave) * E + e] = cnt;
    }
  }
}

__global__ __launch_bounds__(256) void aux_final_kernel(const float* __restrict__ part_prob,
                                                        const int32_t* __restrict__ part_cnt,
                                                        float* __restrict__ l_aux,
                                                        float* __restrict__ mean_prob,
                                                        int32_t* __restrict__ first_counts,
                                                        int n_waves, int T, int E) {
  __shared__ float term[kMaxExperts];
  for (int e = threadIdx.x; e < E; e += blockDim.x) {
    float prob = 0.f;
    int cnt = 0;
    for (int w = 0; w < n_waves; ++w) {
      prob += part_prob[static_cast<size_t>(w) * E + e];
      cnt += part_cnt[static_cast<size_t>(w) * E + e];
    }
    const float mp = T > 0 ? prob / static_cast<float>(T) : 0.f;
    if (mean_prob != nullptr) mean_prob[e] = mp;
    if (first_counts != nullptr) first_counts[e] = cnt;
    term[e] = T > 0 ? mp * (static_cast<float>(cnt) / static_cast<float>(T)) : 0.f;
  }
  __syncthreads();
  if (threadIdx.x == 0) {
    float s = 0.f;
    for (int e = 0; e < E; ++e) s += term[e];   // ascending expert order
    *l_aux = static_cast<float>(E) * s;
  }
}

size_t aux_scratch_bytes(const moe_config& c) {
  const size_t n_waves = (static_cast<size_t>(c.T) + kWave - 1) / kWave;
  return n_waves * c.E * (sizeof(float) + sizeof(int32_t)) + 256;
}

hipError_t launch_aux_loss(const moe_config& c, const float* logits, const int32_t* expert_idx,
                           float* l_aux, float* mean_prob, int32_t* first_counts, void* scratch,
                           hipStream_t s) {
  const int n_waves = (c.T + kWave - 1) / kWave;
  float* part_prob = static_cast<float*>(scratch);
  int32_t* part_cnt = reinterpret_cast<int32_t*>(part_prob + static_cast<size_t>(n_waves) * c.E);
  if (n_waves > 0)
    aux_partial_kernel<<<(n_waves + 3) / 4, 256, 0, s>>>(logits, expert_idx, part_prob, part_cnt, c.T,
                                                         c.E, c.top_k);
  aux_final_kernel<<<1, 256, 0, s>>>(part_prob, part_cnt, l_aux, mean_prob, first_counts, n_waves,
                                     c.T, c.E);
  return hipGetLastError();
}

}  // namespace ppmoe
