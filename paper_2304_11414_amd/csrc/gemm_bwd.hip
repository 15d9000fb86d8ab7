// Backward of the local experts' FFN (Section 3.2, footnote to Eq. 1: the backward pass costs about
// twice the forward; the paper trains through automatic differentiation and prints no algorithm, so
// this is the chain rule of  U = X A,  H = GeLU(U),  Y = H B  per expert):
//
//   dH = dY B^T,   dU = dH * GeLU'(U),   dX = dU A^T,   dA = X^T dU,   dB = H^T dY.
//
// With the library's [out, in] weight layout (W1[i] = A_i^T: [F, d]; W2[i] = B_i^T: [d, F]) the two
// data gradients are products with a weight matrix whose CONTRACTION index is its row index
//   dH[r, f] = sum_c dY[r, c] W2[i][c, f],        dX[r, c] = sum_f dU[r, f] W1[i][f, c],
// and the two weight gradients contract over the packed rows of the expert
//   dW2[i][c, f] = sum_r dY[r, c] H[r, f],        dW1[i][f, c] = sum_r dU[r, f] X[r, c],
// so in both an operand reaches the matrix cores across its rows.  One kernel covers the two forms:
// 128 x 128 x 32 block tile, four wavefronts (2 x 2), each 64 x 64 as 2 x 2 MFMA 32x32x16; operand
// tiles go through LDS as [row][k] with k contiguous (rows 80 bytes apart: the 16 rows a
// ds_read_b128 serves per cycle fall into different banks); an operand whose k runs along memory
// rows is transposed on its way into LDS (16-byte global loads of 8 consecutive rows-of-the-tile at
// one k, eight 2-byte LDS stores).  Weight gradients are float32 (the precision gradients are
// accumulated in); data gradients have the layer's 16-bit type.  Sums have a fixed order: bitwise
// reproducible.

#include "common.h"

namespace ppmoe {

namespace bwd {

constexpr int BM = 128, BN = 128, BK = 32;
constexpr int kThreads = 256;
constexpr int kRowBytes = 80;                 // one tile row in LDS: 32 k-values (64 bytes) + 16 bytes of skew
constexpr int kTileBytes = BM * kRowBytes;    // 10 KiB per operand tile
constexpr int kStages = 2;

// What one operand tile looks like in memory.  `base` points at element (tile row 0, k = 0).
// row_major_k: k is contiguous (element (row, k) at base + row * ld + k); else the tile row index is
// contiguous (element (row, k) at base + k * ld + row).  rows / ks: how many tile rows / k values
// are valid from base on (the rest reads as zero).
struct Operand {
  const bf16_t* base;
  int64_t ld;
  int rows, ks;
};

// Stage one 128 x 32 operand tile (k-tile starting at k0) into registers: 2 pieces of 16 bytes per thread.
template <bool K_CONTIGUOUS>
__device__ __forceinline__ void load_tile(const Operand& op, int k0, u32x4 (&v)[2]) {
  const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int p = threadIdx.x + i * kThreads;
    if (K_CONTIGUOUS) {
      const int row = p >> 2, kc = (p & 3) * 8;   // 4 pieces per row
      const bool ok = row < op.rows && k0 + kc < op.ks;
      v[i] = ok ? *reinterpret_cast<const u32x4*>(op.base + row * op.ld + k0 + kc) : zero;
    } else {
      const int k = p >> 4, rc = (p & 15) * 8;    // 16 pieces per memory row (one k)
      const bool ok = k0 + k < op.ks && rc < op.rows;
      v[i] = ok ? *reinterpret_cast<const u32x4*>(op.base + (k0 + k) * op.ld + rc) : zero;
    }
  }
}

template <bool K_CONTIGUOUS>
__device__ __forceinline__ void store_tile(unsigned char* lds_tile, const u32x4 (&v)[2]) {
#pragma unroll
  for (int i = 0; i < 2; ++i) {
    const int p = threadIdx.x + i * kThreads;
    if (K_CONTIGUOUS) {
      const int row = p >> 2, kc = p & 3;
      *reinterpret_cast<u32x4*>(lds_tile + row * kRowBytes + kc * 16) = v[i];
    } else {
      const int k = p >> 4, rc = (p & 15) * 8;
      const uint32_t w[4] = {v[i].x, v[i].y, v[i].z, v[i].w};
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const uint16_t e = static_cast<uint16_t>(w[j >> 1] >> ((j & 1) * 16));
        *reinterpret_cast<uint16_t*>(lds_tile + (rc + j) * kRowBytes + k * 2) = e;
      }
    }
  }
}

// MODE 0 (data gradient):   C[r, n]    = sum_k A[r, k] * B[i][k, n]   for the rows r of expert i
//                           A [rows, K] 16-bit, B [n_exp, K, N] 16-bit, C [rows, N] 16-bit
// MODE 1 (weight gradient): C[i][m, n] = sum_{r in expert i} A[r, m] * B[r, n]
//                           A [rows, M] 16-bit, B [rows, N] 16-bit, C [n_exp, M, N] float32
template <int MODE, int DT>
__global__ __launch_bounds__(kThreads) void grouped_gemm_bwd_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, void* __restrict__ C,
    const int32_t* __restrict__ offsets, int n_exp, int M, int N, int K) {
  __shared__ __attribute__((aligned(16))) unsigned char lds[kStages * 2 * kTileBytes];
  typedef typename Elem16<DT>::vec8 vec8;

  // ---- which tile ---------------------------------------------------------------------------------
  const int n_tiles = (N + BN - 1) / BN;
  int expert = 0, row0 = 0, rows = 0, col0 = 0, m0 = 0;
  Operand opA, opB;   // opA: the operand whose tile rows are the output rows; opB: the output columns
  int kt_count = 0;
  if (MODE == 0) {
    // tiles ordered expert-major, then n-tile, then m-tile; blocks past the last tile leave
    int tile = blockIdx.x;
    bool found = false;
    int lo = offsets[0];
    for (int i = 0; i < n_exp && !found; ++i) {
      const int hi = offsets[i + 1];
      const int m_tiles = (hi - lo + BM - 1) / BM;
      const int here = m_tiles * n_tiles;
      if (tile < here) {
        const int nt = tile / m_tiles, mt = tile - nt * m_tiles;
        expert = i;
        row0 = lo + mt * BM;
        rows = min(BM, hi - row0);
        col0 = nt * BN;
        found = true;
      } else {
        tile -= here;
        lo = hi;
      }
    }
    if (!found) return;
    opA = Operand{A + static_cast<int64_t>(row0) * K, K, rows, K};
    opB = Operand{B + static_cast<int64_t>(expert) * K * N + col0, N, min(BN, N - col0), K};
    kt_count = (K + BK - 1) / BK;
  } else {
    const int m_tiles = (M + BM - 1) / BM;
    int tile = blockIdx.x;
    expert = tile / (m_tiles * n_tiles);
    tile -= expert * m_tiles * n_tiles;
    const int mt = tile / n_tiles, nt = tile - mt * n_tiles;
    m0 = mt * BM;
    col0 = nt * BN;
    const int lo = offsets[expert], hi = offsets[expert + 1];
    rows = min(BM, M - m0);
    // the contraction runs over the expert's packed rows: k = r - lo
    opA = Operand{A + static_cast<int64_t>(lo) * M + m0, M, rows, hi - lo};
    opB = Operand{B + static_cast<int64_t>(lo) * N + col0, N, min(BN, N - col0), hi - lo};
    kt_count = (hi - lo + BK - 1) / BK;
  }
  constexpr bool kAContig = MODE == 0;   // A[r, k]: k contiguous only for the data gradient
  constexpr bool kBContig = false;       // B's k always runs along memory rows

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 1, wn = wave & 1;
  const int frow = lane & 31, half = lane >> 5;

  f32x16 acc[2][2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

  u32x4 ga[2], gb[2];
  if (kt_count > 0) {
    load_tile<kAContig>(opA, 0, ga);
    load_tile<kBContig>(opB, 0, gb);
    store_tile<kAContig>(lds, ga);
    store_tile<kBContig>(lds + kTileBytes, gb);
  }
  __syncthreads();
  for (int kt = 0; kt < kt_count; ++kt) {
    unsigned char* cur = lds + (kt & 1) * (2 * kTileBytes);
    unsigned char* nxt = lds + ((kt + 1) & 1) * (2 * kTileBytes);
    if (kt + 1 < kt_count) {
      load_tile<kAContig>(opA, (kt + 1) * BK, ga);
      load_tile<kBContig>(opB, (kt + 1) * BK, gb);
    }
#pragma unroll
    for (int ks = 0; ks < 2; ++ks) {
      vec8 fa[2], fb[2];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
        fa[mi] = *reinterpret_cast<const vec8*>(cur + (wm * 64 + mi * 32 + frow) * kRowBytes + ks * 32 + half * 16);
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
        fb[ni] = *reinterpret_cast<const vec8*>(cur + kTileBytes + (wn * 64 + ni * 32 + frow) * kRowBytes + ks * 32 + half * 16);
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
          acc[mi][ni] = Elem16<DT>::mfma32(fb[ni], fa[mi], acc[mi][ni]);   // D[n][m]: lane = row m, registers = columns n
    }
    if (kt + 1 < kt_count) {
      store_tile<kAContig>(nxt, ga);
      store_tile<kBContig>(nxt + kTileBytes, gb);
    }
    __syncthreads();
  }

  // ---- epilogue: lane holds output row m = lane & 31 of each 32-row block and, in register v, column
  // n = (v / 4) * 8 + (lane >> 5) * 4 + v % 4: four consecutive columns per group.
  const int cols = min(BN, N - col0);
#pragma unroll
  for (int mi = 0; mi < 2; ++mi) {
    const int m = wm * 64 + mi * 32 + frow;
    if (m >= rows) continue;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = wn * 64 + ni * 32 + q * 8 + half * 4;
        if (n >= cols) continue;   // (N is a multiple of 8: a group of 4 columns is all in or all out)
        const float v0 = acc[mi][ni][q * 4 + 0], v1 = acc[mi][ni][q * 4 + 1];
        const float v2 = acc[mi][ni][q * 4 + 2], v3 = acc[mi][ni][q * 4 + 3];
        if (MODE == 0) {
          bf16_t* c = static_cast<bf16_t*>(C) + static_cast<int64_t>(row0 + m) * N + col0 + n;
          uint2 p;
          p.x = Elem16<DT>::pack2(v0, v1);
          p.y = Elem16<DT>::pack2(v2, v3);
          *reinterpret_cast<uint2*>(c) = p;
        } else {
          float* c = static_cast<float*>(C) + (static_cast<int64_t>(expert) * M + m0 + m) * N + col0 + n;
          *reinterpret_cast<float4*>(c) = make_float4(v0, v1, v2, v3);
        }
      }
    }
  }
}

// H = GeLU(U) and dU = dH * GeLU'(U), elementwise over the packed rows [0, offsets[n_exp]) x F; dH and
// dU may be the same buffer.  tanh form:  s = 1 / (1 + exp(-2 z)),  z = sqrt(2/pi) (u + 0.044715 u^3):
// GeLU = u s,   GeLU' = s + 2 u s (1 - s) sqrt(2/pi) (1 + 3 * 0.044715 u^2).
template <int DT>
__global__ __launch_bounds__(256) void act_backward_kernel(const bf16_t* __restrict__ U, const bf16_t* dH,
                                                           bf16_t* __restrict__ H, bf16_t* dU,
                                                           const int32_t* __restrict__ offsets, int n_exp,
                                                           int F) {
  const int64_t total = static_cast<int64_t>(offsets[n_exp]) * F / 8;   // 16-byte pieces
  const int64_t stride = static_cast<int64_t>(gridDim.x) * blockDim.x;
  for (int64_t i = static_cast<int64_t>(blockIdx.x) * blockDim.x + threadIdx.x; i < total; i += stride) {
    const u32x4 u4 = reinterpret_cast<const u32x4*>(U)[i];
    const u32x4 g4 = reinterpret_cast<const u32x4*>(dH)[i];
    const uint32_t uw[4] = {u4.x, u4.y, u4.z, u4.w}, gw[4] = {g4.x, g4.y, g4.z, g4.w};
    uint32_t hw[4], dw[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float u[2], g[2], h[2], du[2];
      Elem16<DT>::widen2(uw[j], u[0], u[1]);
      Elem16<DT>::widen2(gw[j], g[0], g[1]);
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const float z2 = 1.5957691216057308f * u[e] * fmaf(0.044715f * u[e], u[e], 1.0f);   // 2 z
        const float s = 1.0f / (1.0f + __expf(-z2));
        h[e] = u[e] * s;
        const float dz2 = 1.5957691216057308f * fmaf(3.0f * 0.044715f * u[e], u[e], 1.0f);  // d(2 z)/du
        du[e] = g[e] * (s + h[e] * (1.0f - s) * dz2);
      }
      hw[j] = Elem16<DT>::pack2(h[0], h[1]);
      dw[j] = Elem16<DT>::pack2(du[0], du[1]);
    }
    reinterpret_cast<u32x4*>(H)[i] = u32x4{hw[0], hw[1], hw[2], hw[3]};
    reinterpret_cast<u32x4*>(dU)[i] = u32x4{dw[0], dw[1], dw[2], dw[3]};
  }
}

}  // namespace bwd

size_t expert_ffn_backward_scratch_bytes(const moe_config& c, int64_t rows) {
  // U, H, dU: three [rows, F] 16-bit buffers (256-byte aligned), then the forward GEMM's scratch
  const size_t one = (static_cast<size_t>(rows) * c.F * 2 + 255) & ~size_t(255);
  return 3 * one + grouped_gemm_workspace_bytes();
}

hipError_t launch_expert_ffn_backward(const moe_config& c, int64_t rows, const void* x_sliced,
                                      const int32_t* offsets, const void* W1, const void* W2,
                                      const void* dY, void* dX, float* dW1, float* dW2, void* scratch,
                                      hipStream_t s) {
  using namespace bwd;
  // (rows == 0: no packed row can exist; every launch below is then empty except the two weight
  // gradients, whose tiles store zeros)
  const size_t one = (static_cast<size_t>(rows) * c.F * 2 + 255) & ~size_t(255);
  unsigned char* ws = static_cast<unsigned char*>(scratch);
  bf16_t* U = reinterpret_cast<bf16_t*>(ws);
  bf16_t* H = reinterpret_cast<bf16_t*>(ws + one);
  bf16_t* dU = reinterpret_cast<bf16_t*>(ws + 2 * one);
  void* gemm_ws = ws + 3 * one;
  const int N = c.local_count;
  const bf16_t* xs = static_cast<const bf16_t*>(x_sliced);
  const bf16_t* w1 = static_cast<const bf16_t*>(W1);
  const bf16_t* w2 = static_cast<const bf16_t*>(W2);
  const bf16_t* dy = static_cast<const bf16_t*>(dY);

  // U = X A (the forward's first GEMM without its activation)
  hipError_t e = launch_grouped_gemm(c.in_dtype, false, x_sliced, W1, U, offsets, N, rows, c.F, c.d, gemm_ws, s);
  if (e != hipSuccess) return e;

  auto dgrad_grid = [&](int n_out) {
    const int64_t m_tiles = (rows + BM - 1) / BM + N;   // upper bound on the sum of the ceilings
    return static_cast<unsigned>(m_tiles * ((n_out + BN - 1) / BN));
  };
  auto wgrad_grid = [&](int m_out, int n_out) {
    return static_cast<unsigned>(static_cast<int64_t>(N) * ((m_out + BM - 1) / BM) * ((n_out + BN - 1) / BN));
  };
#define PPMOE_BWD(MODE, grid, a, b, cc, m, n, k)                                                       \
  do {                                                                                                 \
    if (c.in_dtype == MOE_F16)                                                                         \
      grouped_gemm_bwd_kernel<MODE, MOE_F16><<<grid, kThreads, 0, s>>>(a, b, cc, offsets, N, m, n, k);  \
    else                                                                                               \
      grouped_gemm_bwd_kernel<MODE, MOE_BF16><<<grid, kThreads, 0, s>>>(a, b, cc, offsets, N, m, n, k); \
  } while (0)

  // dH = dY B^T  (into the dU buffer), then H = GeLU(U), dU = dH * GeLU'(U) in place
  PPMOE_BWD(0, dgrad_grid(c.F), dy, w2, dU, 0, c.F, c.d);
  {
    const int64_t pieces = rows * c.F / 8;
    const int blocks = static_cast<int>(pieces / 256 + 1 < 256 * 8 ? pieces / 256 + 1 : 256 * 8);
    if (c.in_dtype == MOE_F16)
      act_backward_kernel<MOE_F16><<<blocks, 256, 0, s>>>(U, dU, H, dU, offsets, N, c.F);
    else
      act_backward_kernel<MOE_BF16><<<blocks, 256, 0, s>>>(U, dU, H, dU, offsets, N, c.F);
  }
  // dX = dU A^T
  PPMOE_BWD(0, dgrad_grid(c.d), dU, w1, dX, 0, c.d, c.F);
  // dB^T[i] = dY_i^T H_i  ([d, F]);  dA^T[i] = dU_i^T X_i  ([F, d])
  PPMOE_BWD(1, wgrad_grid(c.d, c.F), dy, H, dW2, c.d, c.F, 0);
  PPMOE_BWD(1, wgrad_grid(c.F, c.d), dU, xs, dW1, c.F, c.d, 0);
#undef PPMOE_BWD
  return hipGetLastError();
}

}  // namespace ppmoe
