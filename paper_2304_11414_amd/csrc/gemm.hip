// Grouped expert GEMMs (Section 3.3.2: the N local experts of a device; FFN = GeLU(X A) B,
// Section 3.1.3).  The paper runs its experts one after another; here all local experts are one
// launch: the packed rows [offsets[i], offsets[i+1]) of A multiply expert i's weight matrix.
//
//   C[r, n] = act( sum_k A[r, k] * B[i][n, k] )      A [rows, K], B [n_exp, Nout, K], C [rows, Nout]
//
// Both operands are K-contiguous, so every global access is a 16-byte piece of a row.
//
// bf16 kernel: 256x256x64 block tile, 8 wavefronts (2 along rows x 4 along columns), each owning a
// 128x64 sub-tile as 4x2 MFMA 32x32x16 accumulators (128 VGPRs).  Tiles are staged through LDS,
// double buffered, with an XOR swizzle of the 16-byte pieces so that both the row-wise stores and
// the column-of-rows MFMA operand reads are conflict free.  The MFMA computes C^T (weights as the
// A operand, tokens as the B operand) so that each lane ends up with 4 consecutive output columns
// of one row and can store them as one 8-byte piece.
//
// The tile list is built on the device from offsets[]: a block decodes its (expert, m-tile, n-tile)
// from blockIdx, blocks beyond the real tile count exit at once.  No host round trip.

#include "common.h"

namespace ppmoe {


__device__ __forceinline__ float gelu_tanh_fast(float u) {
  // 0.5 u (1 + tanh(z)) = u / (1 + exp(-2 z)),  z = sqrt(2/pi) (u + 0.044715 u^3)
  const float z2 = 1.5957691216057308f * u * fmaf(0.044715f * u, u, 1.0f);
  return u / (1.0f + __expf(-z2));
}

__device__ __forceinline__ float gelu_tanh_precise(float u) {
  const float z = 0.7978845608028654f * u * fmaf(0.044715f * u, u, 1.0f);
  return 0.5f * u * (1.0f + tanhf(z));
}

// Decode a linear tile id into (expert, first row, rows in tile, first column).  Tiles are ordered
// expert-major, then n-tile, then m-tile (m fastest): blocks that run together share a weight panel.
struct TileCoord {
  int expert, row0, rows, col0;
  bool valid;
};

template <int BM, int BN>
__device__ __forceinline__ TileCoord decode_tile(const int32_t* __restrict__ offsets, int n_exp,
                                                 int Nout, int tile) {
  TileCoord tc;
  tc.valid = false;
  tc.expert = tc.row0 = tc.rows = tc.col0 = 0;
  const int n_tiles = (Nout + BN - 1) / BN;
  int lo = offsets[0];
  for (int i = 0; i < n_exp; ++i) {
    const int hi = offsets[i + 1];
    const int m_tiles = (hi - lo + BM - 1) / BM;
    const int here = m_tiles * n_tiles;
    if (tile < here) {
      const int nt = tile / m_tiles, mt = tile - nt * m_tiles;
      tc.expert = i;
      tc.row0 = lo + mt * BM;
      tc.rows = min(BM, hi - tc.row0);
      tc.col0 = nt * BN;
      tc.valid = true;
      return tc;
    }
    tile -= here;
    lo = hi;
  }
  return tc;
}

template <int BM>
__device__ __forceinline__ int total_m_tiles(const int32_t* __restrict__ offsets, int n_exp) {
  int total = 0;
  for (int i = 0; i < n_exp; ++i) total += (offsets[i + 1] - offsets[i] + BM - 1) / BM;
  return total;
}

// Consecutive block ids land on different XCDs (round robin over 8).  Remap so that each XCD works
// on a contiguous run of the tile list and its L2 sees the same weight panel from many CUs.
__device__ __forceinline__ int xcd_remap(int bid, int total) {
  const int per = (total + 7) >> 3;
  const int t = (bid & 7) * per + (bid >> 3);
  return ((bid >> 3) < per && t < total) ? t : -1;
}

// ---------------------------------------------------------------------------------------------
// bf16 MFMA kernel
// ---------------------------------------------------------------------------------------------

constexpr int kBM = 256, kBN = 256, kBK = 64;
constexpr int kGemmThreads = 512;
constexpr int kTileBytes = kBM * kBK * 2;  // one operand tile in LDS: 32 KiB

// Byte offset of 16-byte piece `ch` (0..7) of row `row` inside a tile: rows are 128 bytes, pieces are
// XOR-swizzled with the row number.
__device__ __forceinline__ int lds_piece(int row, int ch) { return row * 128 + ((ch ^ ((row >> 1) & 7)) << 4); }

template <bool GELU, int DT>
__global__ __launch_bounds__(kGemmThreads) void grouped_gemm_bf16_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, bf16_t* __restrict__ C,
    const int32_t* __restrict__ offsets, int n_exp, int Nout, int K) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];  // 2 stages x (A tile + B tile)

  const int n_tiles = (Nout + kBN - 1) / kBN;
  const int total = total_m_tiles<kBM>(offsets, n_exp) * n_tiles;
  const int tile = xcd_remap(blockIdx.x, total);
  if (tile < 0) return;
  const TileCoord tc = decode_tile<kBM, kBN>(offsets, n_exp, Nout, tile);
  if (!tc.valid) return;

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int wm = wave >> 2, wn = wave & 3;  // 2 x 4 wavefronts

  // ---- global -> LDS staging: 2048 pieces per operand tile, 4 per thread --------------------
  const bf16_t* Ab = A + static_cast<size_t>(tc.row0) * K;
  const bf16_t* Bb = B + (static_cast<size_t>(tc.expert) * Nout + tc.col0) * K;
  const int cols = min(kBN, Nout - tc.col0);
  int a_off[4], b_off[4], l_off[4];
  const int ch = tid & 7;
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int row = (tid >> 3) + i * 64;
    a_off[i] = min(row, tc.rows - 1) * K + ch * 8;   // rows past the group re-read its last row
    b_off[i] = min(row, cols - 1) * K + ch * 8;
    l_off[i] = lds_piece(row, ch);
  }
  const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
  u32x4 ga[4], gb[4];
  auto load_global = [&](int k0) {
    const bool ok = k0 + ch * 8 < K;
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      ga[i] = ok ? *reinterpret_cast<const u32x4*>(Ab + a_off[i] + k0) : zero;
      gb[i] = ok ? *reinterpret_cast<const u32x4*>(Bb + b_off[i] + k0) : zero;
    }
  };
  auto store_lds = [&](int stage) {
    unsigned char* base = lds + stage * (2 * kTileBytes);
#pragma unroll
    for (int i = 0; i < 4; ++i) {
      *reinterpret_cast<u32x4*>(base + l_off[i]) = ga[i];
      *reinterpret_cast<u32x4*>(base + kTileBytes + l_off[i]) = gb[i];
    }
  };

  // ---- MFMA operand addressing ---------------------------------------------------------------
  // Lane holds row (lane % 32) of a 32-row fragment and the 8 k-values of piece 2*ks + lane / 32.
  const int frow = lane & 31, half = lane >> 5;
  int tok_base = lds_piece(wm * 128 + frow, 0) & ~127;   // row start; piece added per k-step
  int wgt_base = kTileBytes + (lds_piece(wn * 64 + frow, 0) & ~127);
  int piece[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) piece[ks] = ((2 * ks + half) ^ ((frow >> 1) & 7)) << 4;

  f32x16 acc[4][2];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int ni = 0; ni < 2; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

  const int KT = (K + kBK - 1) / kBK;
  load_global(0);
  store_lds(0);
  __syncthreads();

  for (int kt = 0; kt < KT; ++kt) {
    const int stage = kt & 1;
    if (kt + 1 < KT) load_global((kt + 1) * kBK);
    const unsigned char* base = lds + stage * (2 * kTileBytes);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      typedef typename Elem16<DT>::vec8 vec8;
      vec8 tok[4], wgt[2];
#pragma unroll
      for (int mi = 0; mi < 4; ++mi)
        tok[mi] = *reinterpret_cast<const vec8*>(base + tok_base + mi * (32 * 128) + piece[ks]);
#pragma unroll
      for (int ni = 0; ni < 2; ++ni)
        wgt[ni] = *reinterpret_cast<const vec8*>(base + wgt_base + ni * (32 * 128) + piece[ks]);
#pragma unroll
      for (int mi = 0; mi < 4; ++mi)
#pragma unroll
        for (int ni = 0; ni < 2; ++ni)
          acc[mi][ni] = Elem16<DT>::mfma32(wgt[ni], tok[mi], acc[mi][ni]);
    }
    if (kt + 1 < KT) store_lds(stage ^ 1);
    __syncthreads();
  }

  // ---- epilogue ------------------------------------------------------------------------------
  // D = W_frag (32 n) x Tok_frag^T (32 m): lane holds token column m = lane % 32 and, in register
  // v, output column n = (v / 4) * 8 + (lane / 32) * 4 + v % 4.
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) {
    const int m = wm * 128 + mi * 32 + frow;
    if (m >= tc.rows) continue;
    bf16_t* crow = C + static_cast<size_t>(tc.row0 + m) * Nout + tc.col0;
#pragma unroll
    for (int ni = 0; ni < 2; ++ni) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = wn * 64 + ni * 32 + q * 8 + half * 4;
        if (n >= cols) continue;
        float v0 = acc[mi][ni][q * 4 + 0], v1 = acc[mi][ni][q * 4 + 1];
        float v2 = acc[mi][ni][q * 4 + 2], v3 = acc[mi][ni][q * 4 + 3];
        if (GELU) {
          v0 = gelu_tanh_fast(v0);
          v1 = gelu_tanh_fast(v1);
          v2 = gelu_tanh_fast(v2);
          v3 = gelu_tanh_fast(v3);
        }
        uint2 p;
        p.x = Elem16<DT>::pack2(v0, v1);
        p.y = Elem16<DT>::pack2(v2, v3);
        *reinterpret_cast<uint2*>(crow + n) = p;
      }
    }
  }
}

// ---------------------------------------------------------------------------------------------
// float32 kernel (the small parity configuration): 64x64x16 tiles, 4x4 outputs per thread, plain
// FMA, precise tanh.
// ---------------------------------------------------------------------------------------------

constexpr int kFM = 64, kFN = 64, kFK = 16;

template <bool GELU>
__global__ __launch_bounds__(256) void grouped_gemm_f32_kernel(
    const float* __restrict__ A, const float* __restrict__ B, float* __restrict__ C,
    const int32_t* __restrict__ offsets, int n_exp, int Nout, int K) {
  __shared__ float As[kFK][kFM + 4];
  __shared__ float Bs[kFK][kFN + 4];
  const int n_tiles = (Nout + kFN - 1) / kFN;
  const int total = total_m_tiles<kFM>(offsets, n_exp) * n_tiles;
  if (static_cast<int>(blockIdx.x) >= total) return;
  const TileCoord tc = decode_tile<kFM, kFN>(offsets, n_exp, Nout, blockIdx.x);
  if (!tc.valid) return;
  const int cols = min(kFN, Nout - tc.col0);
  const float* Ab = A + static_cast<size_t>(tc.row0) * K;
  const float* Bb = B + (static_cast<size_t>(tc.expert) * Nout + tc.col0) * K;

  const int tid = threadIdx.x;
  const int lrow = tid >> 2, lq = tid & 3;          // staging: row 0..63, float4 piece 0..3
  const int ty = tid >> 4, tx = tid & 15;           // compute: 16 x 16 threads, 4x4 outputs each
  const int arow = min(lrow, tc.rows - 1), brow = min(lrow, cols - 1);
  float acc[4][4] = {};
  for (int k0 = 0; k0 < K; k0 += kFK) {
    const int kk = k0 + lq * 4;
    float4 av = make_float4(0.f, 0.f, 0.f, 0.f), bv = av;
    if (kk < K) {  // K is a multiple of 8, so a float4 piece is all-in or all-out
      av = *reinterpret_cast<const float4*>(Ab + static_cast<size_t>(arow) * K + kk);
      bv = *reinterpret_cast<const float4*>(Bb + static_cast<size_t>(brow) * K + kk);
    }
    As[lq * 4 + 0][lrow] = av.x; As[lq * 4 + 1][lrow] = av.y;
    As[lq * 4 + 2][lrow] = av.z; As[lq * 4 + 3][lrow] = av.w;
    Bs[lq * 4 + 0][lrow] = bv.x; Bs[lq * 4 + 1][lrow] = bv.y;
    Bs[lq * 4 + 2][lrow] = bv.z; Bs[lq * 4 + 3][lrow] = bv.w;
    __syncthreads();
#pragma unroll
    for (int k = 0; k < kFK; ++k) {
      float a[4], b[4];
#pragma unroll
      for (int i = 0; i < 4; ++i) a[i] = As[k][ty * 4 + i];
#pragma unroll
      for (int j = 0; j < 4; ++j) b[j] = Bs[k][tx * 4 + j];
#pragma unroll
      for (int i = 0; i < 4; ++i)
#pragma unroll
        for (int j = 0; j < 4; ++j) acc[i][j] = fmaf(a[i], b[j], acc[i][j]);
    }
    __syncthreads();
  }
#pragma unroll
  for (int i = 0; i < 4; ++i) {
    const int m = ty * 4 + i;
    if (m >= tc.rows) continue;
    const int n = tx * 4;
    if (n >= cols) continue;   // Nout is a multiple of 8: a group of 4 columns is all-in or all-out
    float4 v = make_float4(acc[i][0], acc[i][1], acc[i][2], acc[i][3]);
    if (GELU) {
      v.x = gelu_tanh_precise(v.x);
      v.y = gelu_tanh_precise(v.y);
      v.z = gelu_tanh_precise(v.z);
      v.w = gelu_tanh_precise(v.w);
    }
    *reinterpret_cast<float4*>(C + static_cast<size_t>(tc.row0 + m) * Nout + tc.col0 + n) = v;
  }
}

// ---------------------------------------------------------------------------------------------

static hipError_t ensure_lds_attr() {
  static std::atomic<uint64_t> done{0};
  return once_per_device(done, [] {
    const void* kernels[] = {reinterpret_cast<const void*>(grouped_gemm_bf16_kernel<true, MOE_BF16>),
                             reinterpret_cast<const void*>(grouped_gemm_bf16_kernel<false, MOE_BF16>),
                             reinterpret_cast<const void*>(grouped_gemm_bf16_kernel<true, MOE_F16>),
                             reinterpret_cast<const void*>(grouped_gemm_bf16_kernel<false, MOE_F16>)};
    for (const void* k : kernels) {
      hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, 4 * kTileBytes);
      if (e != hipSuccess) return e;
    }
    return hipSuccess;
  });
}

hipError_t launch_grouped_gemm(int in_dtype, bool gelu, const void* A, const void* B, void* C,
                               const int32_t* offsets, int n_exp, int64_t max_rows, int Nout, int K,
                               void* workspace, hipStream_t s, int fuse, const int32_t* aux_rows,
                               const float* aux_w, int aux_div, const int32_t* aux_inv, void* C2) {
  if (max_rows == 0) return hipSuccess;
  if (grouped_gemm_is_fast(in_dtype, K)) {
    return launch_grouped_gemm_fast(in_dtype, gelu, static_cast<const bf16_t*>(A), static_cast<const bf16_t*>(B),
                                    static_cast<bf16_t*>(C), offsets, n_exp, max_rows, Nout, K, workspace, s,
                                    fuse, aux_rows, aux_w, aux_div, aux_inv, static_cast<bf16_t*>(C2));
  }
  if (fuse != 0) return hipErrorInvalidValue;   // the other kernels work on packed tensors only
  if (is_16bit(in_dtype)) {
    hipError_t e = ensure_lds_attr();
    if (e != hipSuccess) return e;
    const int64_t m_tiles = (max_rows + kBM - 1) / kBM + n_exp;   // upper bound on sum of ceilings
    const int64_t n_tiles = (Nout + kBN - 1) / kBN;
    const int64_t grid = ((m_tiles * n_tiles + 7) / 8) * 8;
    const bf16_t* a = static_cast<const bf16_t*>(A);
    const bf16_t* b = static_cast<const bf16_t*>(B);
    bf16_t* c = static_cast<bf16_t*>(C);
#define PPMOE_GEMM16(G, DT)                                                                         \
  grouped_gemm_bf16_kernel<G, DT><<<static_cast<unsigned>(grid), kGemmThreads, 4 * kTileBytes, s>>>( \
      a, b, c, offsets, n_exp, Nout, K)
    if (in_dtype == MOE_F16) {
      if (gelu) PPMOE_GEMM16(true, MOE_F16);
      else PPMOE_GEMM16(false, MOE_F16);
    } else {
      if (gelu) PPMOE_GEMM16(true, MOE_BF16);
      else PPMOE_GEMM16(false, MOE_BF16);
    }
#undef PPMOE_GEMM16
  } else {
    const int64_t m_tiles = (max_rows + kFM - 1) / kFM + n_exp;
    const int64_t n_tiles = (Nout + kFN - 1) / kFN;
    const int64_t grid = m_tiles * n_tiles;
    const float* a = static_cast<const float*>(A);
    const float* b = static_cast<const float*>(B);
    float* c = static_cast<float*>(C);
    if (gelu)
      grouped_gemm_f32_kernel<true><<<static_cast<unsigned>(grid), 256, 0, s>>>(a, b, c, offsets, n_exp, Nout, K);
    else
      grouped_gemm_f32_kernel<false><<<static_cast<unsigned>(grid), 256, 0, s>>>(a, b, c, offsets, n_exp, Nout, K);
  }
  return hipGetLastError();
}

}  // namespace ppmoe
