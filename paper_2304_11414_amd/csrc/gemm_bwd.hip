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
// 128 x 128 x 64 block tile, four wavefronts (2 x 2), each 64 x 64 as 2 x 2 MFMA 32x32x16; operand
// tiles go through LDS as [row][k] with k contiguous (rows 144 bytes apart, 16-byte chunks
// XOR-swizzled: fragment reads and staging writes are free of bank conflicts); an operand whose k
// runs along memory rows is transposed in registers on its way into LDS (a thread loads an 8 x 8
// block as eight 16-byte pieces, one per memory row, and writes eight 16-byte chunks, one per tile
// row).  Weight gradients are float32 (the precision gradients are accumulated in); data gradients
// have the layer's 16-bit type.  Sums have a fixed order: bitwise reproducible.

#include "common.h"

namespace ppmoe {

namespace bwd {

constexpr int BM = 128, BN = 128, BK = 64;
constexpr int kThreads = 256;
constexpr int kRowBytes = 144;                // one tile row in LDS: 64 k-values (128 bytes) + 16 bytes of skew
constexpr int kTileBytes = BM * kRowBytes;    // 18 KiB per operand tile
constexpr int kStages = 2;
constexpr int kLdsBytes = kStages * 2 * kTileBytes;   // 72 KiB

// Byte offset of 16-byte chunk `ch` (8 k-values) of tile row `row`: chunks are XOR-swizzled with the
// row's group of 16, so that the eight rows a thread writes after its in-register transpose, 16 rows
// apart from the next lane's, and the 16 consecutive rows a fragment read serves per cycle both
// spread over all banks.
__device__ __forceinline__ int lds_chunk(int row, int ch) {
  return row * kRowBytes + ((ch ^ ((row >> 4) & 7)) << 4);
}

// What one operand tile looks like in memory.  `base` points at element (tile row 0, k = 0).
// K-contiguous: element (row, k) at base + row * ld + k; else the tile row index is contiguous:
// element (row, k) at base + k * ld + row.  rows / ks: how many tile rows / k values are valid from
// base on (the rest reads as zero).
struct Operand {
  const bf16_t* base;
  int64_t ld;
  int rows, ks;
};

// One operand tile is 128 rows x 64 k = 1024 chunks of 16 bytes, staged by two wavefronts (half: which
// of the two), eight chunks per thread.
//  * k contiguous in memory: lane = (row % 8) * 8 + chunk; eight lanes read one whole 128-byte line.
//  * rows contiguous in memory: a thread reads an 8 (k) x 8 (rows) block, one 16-byte piece from each
//    of eight consecutive memory rows (16 lanes read 256 contiguous bytes of each), transposes it in
//    registers (v_perm_b32) and writes eight 16-byte chunks, one per tile row.
template <bool K_CONTIGUOUS>
__device__ __forceinline__ void load_tile(const Operand& op, int k0, int half, int lane, u32x4 (&v)[8]) {
  const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
  if (K_CONTIGUOUS) {
    const int ch = lane & 7;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = (lane >> 3) + 8 * half + 16 * i;
      const bool ok = row < op.rows && k0 + ch * 8 < op.ks;
      v[i] = ok ? *reinterpret_cast<const u32x4*>(op.base + row * op.ld + k0 + ch * 8) : zero;
    }
  } else {
    const int rg = lane & 15, kg = half * 4 + (lane >> 4);
#pragma unroll
    for (int kk = 0; kk < 8; ++kk) {
      const int k = k0 + kg * 8 + kk;
      const bool ok = k < op.ks && rg * 8 < op.rows;
      v[kk] = ok ? *reinterpret_cast<const u32x4*>(op.base + k * op.ld + rg * 8) : zero;
    }
  }
}

template <bool K_CONTIGUOUS>
__device__ __forceinline__ void store_tile(unsigned char* lds_tile, int half, int lane, const u32x4 (&v)[8]) {
  if (K_CONTIGUOUS) {
    const int ch = lane & 7;
#pragma unroll
    for (int i = 0; i < 8; ++i) {
      const int row = (lane >> 3) + 8 * half + 16 * i;
      *reinterpret_cast<u32x4*>(lds_tile + lds_chunk(row, ch)) = v[i];
    }
  } else {
    const int rg = lane & 15, kg = half * 4 + (lane >> 4);
    // v[kk] dword q holds tile rows 2q (low half) and 2q + 1 (high half) at k = kk; the chunk of tile
    // row r wants, in dword q, k = 2q (low) and 2q + 1 (high).
#pragma unroll
    for (int r = 0; r < 8; ++r) {
      u32x4 o;
      const uint32_t sel = (r & 1) ? 0x07060302u : 0x05040100u;
      o.x = __builtin_amdgcn_perm(v[1][r >> 1], v[0][r >> 1], sel);
      o.y = __builtin_amdgcn_perm(v[3][r >> 1], v[2][r >> 1], sel);
      o.z = __builtin_amdgcn_perm(v[5][r >> 1], v[4][r >> 1], sel);
      o.w = __builtin_amdgcn_perm(v[7][r >> 1], v[6][r >> 1], sel);
      *reinterpret_cast<u32x4*>(lds_tile + lds_chunk(rg * 8 + r, kg)) = o;
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
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  typedef typename Elem16<DT>::vec8 vec8;

  // ---- which tile ---------------------------------------------------------------------------------
  const int n_tiles = (N + BN - 1) / BN;
  int expert = 0, row0 = 0, rows = 0, col0 = 0, m0 = 0;
  Operand opA, opB;   // opA: the operand whose tile rows are the output rows; opB: the output columns
  int kt_count = 0;
  // Consecutive block ids land on different XCDs (round robin over 8): remap so that each XCD works on
  // a contiguous run of the tile list and its L2 sees the same panels from many CUs.
  auto xcd_tile = [](int bid, int total) {
    const int per = (total + 7) >> 3;
    const int t = (bid & 7) * per + (bid >> 3);
    return ((bid >> 3) < per && t < total) ? t : -1;
  };
  if (MODE == 0) {
    // tiles ordered expert-major, then n-tile, then m-tile; blocks past the last tile leave
    int total = 0;
    for (int i = 0; i < n_exp; ++i) total += (offsets[i + 1] - offsets[i] + BM - 1) / BM * n_tiles;
    int tile = xcd_tile(blockIdx.x, total);
    if (tile < 0) return;
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
    int tile = xcd_tile(blockIdx.x, n_exp * m_tiles * n_tiles);
    if (tile < 0) return;
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

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int frow = lane & 31, half = lane >> 5;
  // staging: wavefronts 0, 1 bring in the A tile, 2, 3 the B tile
  const bool stage_b = wave >= 2;
  const int stage_half = wave & 1;

  f32x16 acc[2][2];
#pragma unroll
  for (int mi = 0; mi < 2; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

  u32x4 g[8];
  auto load = [&](int kt) {
    if (stage_b) load_tile<false>(opB, kt * BK, stage_half, lane, g);
    else load_tile<kAContig>(opA, kt * BK, stage_half, lane, g);
  };
  auto store = [&](unsigned char* buf) {
    if (stage_b) store_tile<false>(buf + kTileBytes, stage_half, lane, g);
    else store_tile<kAContig>(buf, stage_half, lane, g);
  };
  if (kt_count > 0) {
    load(0);
    store(lds);
  }
  __syncthreads();
  for (int kt = 0; kt < kt_count; ++kt) {
    unsigned char* cur = lds + (kt & 1) * (2 * kTileBytes);
    unsigned char* nxt = lds + ((kt + 1) & 1) * (2 * kTileBytes);
    if (kt + 1 < kt_count) load(kt + 1);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      vec8 fa[2], fb[2];
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
        fa[mi] = *reinterpret_cast<const vec8*>(cur + lds_chunk(wm * 64 + mi * 32 + frow, ks * 2 + half));
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
        fb[ni] = *reinterpret_cast<const vec8*>(cur + kTileBytes + lds_chunk(wn * 64 + ni * 32 + frow, ks * 2 + half));
#pragma unroll
      for (int mi = 0; mi < 2; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
          acc[mi][ni] = Elem16<DT>::mfma32(fb[ni], fa[mi], acc[mi][ni]);   // D[n][m]: lane = row m, registers = columns n
    }
    if (kt + 1 < kt_count) store(nxt);
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

// H = GeLU(U) and dU = dH * GeLU'(U) over the packed rows [0, offsets[n_exp]) x F, one row per block
// iteration; dH and dU may be the same buffer.  tanh form:  s = 1 / (1 + exp(-2 z)),
// z = sqrt(2/pi) (u + 0.044715 u^3):   GeLU = u s,   GeLU' = s + 2 u s (1 - s) sqrt(2/pi) (1 + 3 * 0.044715 u^2).
// row_dot (may be NULL): row_dot[r] = sum_f dH[r, f] * H[r, f], the derivative with respect to a
// scale factor of the row's expert output (what the gate weight's gradient is made of), added up in a
// fixed order (butterfly inside a wavefront, wavefronts in order).
template <int DT>
__global__ __launch_bounds__(256) void act_backward_kernel(const bf16_t* __restrict__ U, const bf16_t* dH,
                                                           bf16_t* __restrict__ H, bf16_t* dU,
                                                           float* __restrict__ row_dot,
                                                           const int32_t* __restrict__ offsets, int n_exp,
                                                           int F) {
  __shared__ float part[4];
  const int rows = offsets[n_exp];
  const int pieces = F / 8;   // 16-byte pieces per row
  for (int r = blockIdx.x; r < rows; r += gridDim.x) {
    float dot = 0.f;
    for (int i = threadIdx.x; i < pieces; i += 256) {
      const int64_t at = static_cast<int64_t>(r) * pieces + i;
      const u32x4 u4 = reinterpret_cast<const u32x4*>(U)[at];
      const u32x4 g4 = reinterpret_cast<const u32x4*>(dH)[at];
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
          const float sg = 1.0f / (1.0f + __expf(-z2));
          h[e] = u[e] * sg;
          const float dz2 = 1.5957691216057308f * fmaf(3.0f * 0.044715f * u[e], u[e], 1.0f);  // d(2 z)/du
          du[e] = g[e] * (sg + h[e] * (1.0f - sg) * dz2);
          dot = fmaf(g[e], h[e], dot);
        }
        hw[j] = Elem16<DT>::pack2(h[0], h[1]);
        dw[j] = Elem16<DT>::pack2(du[0], du[1]);
      }
      reinterpret_cast<u32x4*>(H)[at] = u32x4{hw[0], hw[1], hw[2], hw[3]};
      reinterpret_cast<u32x4*>(dU)[at] = u32x4{dw[0], dw[1], dw[2], dw[3]};
    }
    if (row_dot != nullptr) {   // (uniform)
#pragma unroll
      for (int off = 32; off >= 1; off >>= 1) dot += __shfl_xor(dot, off, 64);
      if ((threadIdx.x & 63) == 0) part[threadIdx.x >> 6] = dot;
      __syncthreads();
      if (threadIdx.x == 0) row_dot[r] = ((part[0] + part[1]) + part[2]) + part[3];
      __syncthreads();
    }
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
                                      hipStream_t s, float* row_dot) {
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
    return static_cast<unsigned>((m_tiles * ((n_out + BN - 1) / BN) + 7) / 8 * 8);
  };
  auto wgrad_grid = [&](int m_out, int n_out) {
    return static_cast<unsigned>((static_cast<int64_t>(N) * ((m_out + BM - 1) / BM) * ((n_out + BN - 1) / BN) + 7) / 8 * 8);
  };
  static const hipError_t attrs = [] {
    const void* kernels[] = {reinterpret_cast<const void*>(grouped_gemm_bwd_kernel<0, MOE_BF16>),
                             reinterpret_cast<const void*>(grouped_gemm_bwd_kernel<1, MOE_BF16>),
                             reinterpret_cast<const void*>(grouped_gemm_bwd_kernel<0, MOE_F16>),
                             reinterpret_cast<const void*>(grouped_gemm_bwd_kernel<1, MOE_F16>)};
    for (const void* k : kernels) {
      hipError_t err = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
      if (err != hipSuccess) return err;
    }
    return hipSuccess;
  }();
  if (attrs != hipSuccess) return attrs;
#define PPMOE_BWD(MODE, grid, a, b, cc, m, n, k)                                                               \
  do {                                                                                                         \
    if (c.in_dtype == MOE_F16)                                                                                 \
      grouped_gemm_bwd_kernel<MODE, MOE_F16><<<grid, kThreads, kLdsBytes, s>>>(a, b, cc, offsets, N, m, n, k);  \
    else                                                                                                       \
      grouped_gemm_bwd_kernel<MODE, MOE_BF16><<<grid, kThreads, kLdsBytes, s>>>(a, b, cc, offsets, N, m, n, k); \
  } while (0)

  // dH = dY B^T  (into the dU buffer), then H = GeLU(U), dU = dH * GeLU'(U) in place
  PPMOE_BWD(0, dgrad_grid(c.F), dy, w2, dU, 0, c.F, c.d);
  {
    const int blocks = static_cast<int>(rows < 256 * 16 ? (rows > 0 ? rows : 1) : 256 * 16);
    if (c.in_dtype == MOE_F16)
      act_backward_kernel<MOE_F16><<<blocks, 256, 0, s>>>(U, dU, H, dU, row_dot, offsets, N, c.F);
    else
      act_backward_kernel<MOE_BF16><<<blocks, 256, 0, s>>>(U, dU, H, dU, row_dot, offsets, N, c.F);
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
