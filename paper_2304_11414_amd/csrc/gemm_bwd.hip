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
// so in both an operand reaches the matrix cores across its rows.  Two kernels cover the two forms
// (MODE 0: data gradient, MODE 1: weight gradient): a hand-scheduled one with 256 x 256 x 64 block
// tiles for launches with enough tiles to fill the chip, and a plain one with 128 x 128 x 64 tiles
// (two blocks per CU, scheduled by the compiler) for everything else.  Both: four wavefronts (2 x 2),
// each a quarter of the tile as MFMA 32x32x16 blocks; operand
// tiles go through LDS as [row][k] with k contiguous (rows 144 bytes apart, 16-byte chunks
// XOR-swizzled: fragment reads and staging writes are free of bank conflicts); an operand whose k
// runs along memory rows is transposed in registers on its way into LDS (a thread loads an 8 x 8
// block as eight 16-byte pieces, one per memory row, and writes eight 16-byte chunks, one per tile
// row).  Weight gradients are float32 (the precision gradients are accumulated in); data gradients
// have the layer's 16-bit type.  Sums have a fixed order: bitwise reproducible.  Where the data
// gradient's contraction is long, the experts' last few rows may leave the 256 x 256 launch for a
// split-contraction launch of their own (tail_threshold below).

#include <type_traits>

#include "common.h"

namespace ppmoe {

namespace bwd {

constexpr int BK = 64;
constexpr int kThreads = 256;
constexpr int kRowBytes = 144;                // one tile row in LDS: 64 k-values (128 bytes) + 16 bytes of skew
constexpr int kStages = 2;
// Block tile BM x BN (each 128 or 256): two stages of (BM + BN) rows; 144 KiB for 256 x 256.
constexpr int lds_bytes(int bm, int bn) { return kStages * (bm + bn) * kRowBytes; }

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

// One operand tile is R rows (128 or 256) x 64 k = 8 R chunks of 16 bytes, staged by two wavefronts
// (half: which of the two), R / 16 chunks per thread.
//  * k contiguous in memory: lane = (row % 8) * 8 + chunk; eight lanes read one whole 128-byte line.
//  * rows contiguous in memory: a thread reads an 8 (k) x 8 (rows) block per group of 128 rows, one
//    16-byte piece from each of eight consecutive memory rows (16 lanes read 256 contiguous bytes of
//    each), transposes it in registers (v_perm_b32) and writes eight 16-byte chunks, one per tile row.
template <bool K_CONTIGUOUS, int R>
__device__ __forceinline__ void load_tile(const Operand& op, int k0, int half, int lane, u32x4* v) {
  const u32x4 zero = u32x4{0u, 0u, 0u, 0u};
  if (K_CONTIGUOUS) {
    const int ch = lane & 7;
#pragma unroll
    for (int i = 0; i < R / 16; ++i) {
      const int row = (lane >> 3) + 8 * half + 16 * i;
      const bool ok = row < op.rows && k0 + ch * 8 < op.ks;
      v[i] = ok ? *reinterpret_cast<const u32x4*>(op.base + row * op.ld + k0 + ch * 8) : zero;
    }
  } else {
    const int rg = lane & 15, kg = half * 4 + (lane >> 4);
#pragma unroll
    for (int g = 0; g < R / 128; ++g) {
#pragma unroll
      for (int kk = 0; kk < 8; ++kk) {
        const int k = k0 + kg * 8 + kk;
        const bool ok = k < op.ks && g * 128 + rg * 8 < op.rows;
        v[g * 8 + kk] = ok ? *reinterpret_cast<const u32x4*>(op.base + k * op.ld + g * 128 + rg * 8) : zero;
      }
    }
  }
}

template <bool K_CONTIGUOUS, int R>
__device__ __forceinline__ void store_tile(unsigned char* lds_tile, int half, int lane, const u32x4* v) {
  if (K_CONTIGUOUS) {
    const int ch = lane & 7;
#pragma unroll
    for (int i = 0; i < R / 16; ++i) {
      const int row = (lane >> 3) + 8 * half + 16 * i;
      *reinterpret_cast<u32x4*>(lds_tile + lds_chunk(row, ch)) = v[i];
    }
  } else {
    const int rg = lane & 15, kg = half * 4 + (lane >> 4);
    // v[g * 8 + kk] dword q holds tile rows 2q (low half) and 2q + 1 (high half) at k = kk; the chunk
    // of tile row r wants, in dword q, k = 2q (low) and 2q + 1 (high).
#pragma unroll
    for (int g = 0; g < R / 128; ++g) {
#pragma unroll
      for (int r = 0; r < 8; ++r) {
        u32x4 o;
        const uint32_t sel = (r & 1) ? 0x07060302u : 0x05040100u;
        o.x = __builtin_amdgcn_perm(v[g * 8 + 1][r >> 1], v[g * 8 + 0][r >> 1], sel);
        o.y = __builtin_amdgcn_perm(v[g * 8 + 3][r >> 1], v[g * 8 + 2][r >> 1], sel);
        o.z = __builtin_amdgcn_perm(v[g * 8 + 5][r >> 1], v[g * 8 + 4][r >> 1], sel);
        o.w = __builtin_amdgcn_perm(v[g * 8 + 7][r >> 1], v[g * 8 + 6][r >> 1], sel);
        *reinterpret_cast<u32x4*>(lds_tile + lds_chunk(g * 128 + rg * 8 + r, kg)) = o;
      }
    }
  }
}

// Which output tile a block computes, and where its operand tiles start.
struct TileInfo {
  int expert, row0, rows, col0, m0, kt_count;
  Operand opA, opB;   // opA: the operand whose tile rows are the output rows; opB: the output columns
};

// Data gradient with a long contraction: an expert's rows past the last multiple of 256 cost the
// 256 x 256 kernel a whole tile each, and with few tiles per CU a whole extra round of the chip.
// They can go to a second launch instead (128-row tiles, 32-row blocks without a valid row skipped,
// the contraction split over several blocks, partial sums added up in a fixed order by a third
// launch).  Every block of the three launches takes that decision from the row counts alone, so they
// all agree.  tail_threshold returns t: remainders of 1..t rows are split off (0: none).  The smaller
// candidate (128) is taken if it saves the 256 x 256 launch at least as much as the larger would;
// a candidate qualifies when what it saves (whole rounds when there are few, else the tiles'
// share of a round) outweighs the tail launch, which runs at about a third of the rate per flop.
constexpr int kTailTile = 128;        // row tile of the tail launch
constexpr int kTailSplitsMax = 8;
__device__ __forceinline__ int tail_rows_of(int n, int threshold) {
  const int t = n & 255;
  return t <= threshold ? t : 0;
}
__device__ __forceinline__ int tail_threshold(const int32_t* __restrict__ offsets, int n_exp, int N, int tail_cus) {
  if (tail_cus <= 0) return 0;   // (the launcher has not provided for the two extra launches)
  const int n_tiles = (N + 255) / 256;
  int all = 0, big[2] = {0, 0}, blocks[2] = {0, 0};   // candidates 128 and 255
  for (int i = 0; i < n_exp; ++i) {
    const int n = offsets[i + 1] - offsets[i];
    all += (n + 255) / 256 * n_tiles;
#pragma unroll
    for (int c = 0; c < 2; ++c) {
      const int t = tail_rows_of(n, c == 0 ? 128 : 255);
      big[c] += (n - t + 255) / 256 * n_tiles;
      blocks[c] += (t + 31) / 32;
    }
  }
  const int rounds_all = (all + tail_cus - 1) / tail_cus;
  int saved[2];
#pragma unroll
  for (int c = 0; c < 2; ++c) {
    // in units of a 32-row block of one 256-column tile: a tile is 8 of them
    const int rounds = (big[c] + tail_cus - 1) / tail_cus;
    const int64_t saving = 8 * (rounds_all <= 4 ? static_cast<int64_t>(rounds_all - rounds) * tail_cus
                                                : static_cast<int64_t>(all - big[c]));
    const int64_t cost = 3 * static_cast<int64_t>(blocks[c]) * n_tiles;
    saved[c] = (all > big[c] && cost <= saving) ? static_cast<int>(saving - cost) + 1 : 0;
  }
  if (saved[0] > 0 && saved[0] >= saved[1]) return 128;
  return saved[1] > 0 ? 255 : 0;
}

// tail_cus (MODE 0 only): 0, or the number of CUs when the launcher runs the tail launches as well.
template <int MODE, int BM, int BN>
__device__ __forceinline__ bool locate_tile(const bf16_t* __restrict__ A, const bf16_t* __restrict__ B,
                                            const int32_t* __restrict__ offsets, int n_exp, int M, int N,
                                            int K, TileInfo& ti, int tail_cus = 0) {
  const int n_tiles = (N + BN - 1) / BN;
  ti.expert = ti.row0 = ti.rows = ti.col0 = ti.m0 = ti.kt_count = 0;
  // Consecutive block ids land on different XCDs (round robin over 8): remap so that each XCD works on
  // a contiguous run of the tile list and its L2 sees the same panels from many CUs.
  auto xcd_tile = [](int bid, int total) {
    const int per = (total + 7) >> 3;
    const int t = (bid & 7) * per + (bid >> 3);
    return ((bid >> 3) < per && t < total) ? t : -1;
  };
  if (MODE == 0) {
    // tiles ordered expert-major, then n-tile, then m-tile; blocks past the last tile leave
    const int tail_thr = tail_threshold(offsets, n_exp, N, tail_cus);
    int total = 0;
    for (int i = 0; i < n_exp; ++i) {
      const int n = offsets[i + 1] - offsets[i];
      total += (n - tail_rows_of(n, tail_thr) + BM - 1) / BM * n_tiles;
    }
    int tile = xcd_tile(blockIdx.x, total);
    if (tile < 0) return false;
    bool found = false;
    int lo = offsets[0];
    for (int i = 0; i < n_exp && !found; ++i) {
      const int next = offsets[i + 1];
      const int hi = next - tail_rows_of(next - lo, tail_thr);
      const int m_tiles = (hi - lo + BM - 1) / BM;
      const int here = m_tiles * n_tiles;
      if (tile < here) {
        const int nt = tile / m_tiles, mt = tile - nt * m_tiles;
        ti.expert = i;
        ti.row0 = lo + mt * BM;
        ti.rows = min(BM, hi - ti.row0);
        ti.col0 = nt * BN;
        found = true;
      } else {
        tile -= here;
        lo = next;
      }
    }
    if (!found) return false;
    ti.opA = Operand{A + static_cast<int64_t>(ti.row0) * K, K, ti.rows, K};
    ti.opB = Operand{B + static_cast<int64_t>(ti.expert) * K * N + ti.col0, N, min(BN, N - ti.col0), K};
    ti.kt_count = (K + BK - 1) / BK;
  } else {
    const int m_tiles = (M + BM - 1) / BM;
    int tile = xcd_tile(blockIdx.x, n_exp * m_tiles * n_tiles);
    if (tile < 0) return false;
    // Tiles ordered in blocks of up to 32 (ba row tiles x bb column tiles of one expert: what the 32
    // CUs of an XCD hold at a time, sharing ba + bb operand panels), the blocks of a position going
    // through all the experts before the next position: each XCD's run of the list visits every
    // expert, so an expert with many rows (a long contraction) is not one XCD's alone.
    int bb = n_tiles % 8 == 0 ? 8 : n_tiles % 4 == 0 ? 4 : n_tiles % 2 == 0 ? 2 : 1;
    int ba = 32 / bb;
    while (ba > 1 && m_tiles % ba != 0) ba >>= 1;
    const int per_block = ba * bb, blocks_n = n_tiles / bb;
    const int blk = tile / (n_exp * per_block);
    tile -= blk * n_exp * per_block;
    ti.expert = tile / per_block;
    const int w = tile - ti.expert * per_block;
    const int mt = (blk / blocks_n) * ba + w / bb, nt = (blk % blocks_n) * bb + w % bb;
    ti.m0 = mt * BM;
    ti.col0 = nt * BN;
    const int lo = offsets[ti.expert], hi = offsets[ti.expert + 1];
    ti.rows = min(BM, M - ti.m0);
    // the contraction runs over the expert's packed rows: k = r - lo
    ti.opA = Operand{A + static_cast<int64_t>(lo) * M + ti.m0, M, ti.rows, hi - lo};
    ti.opB = Operand{B + static_cast<int64_t>(lo) * N + ti.col0, N, min(BN, N - ti.col0), hi - lo};
    ti.kt_count = (hi - lo + BK - 1) / BK;
  }
  return true;
}

// Stores a block's accumulators.  A lane holds output row m = lane & 31 of each 32-row block and, in
// register v, column n = (v / 4) * 8 + (lane >> 5) * 4 + v % 4: four consecutive columns per group.
template <int MODE, int DT, int BM, int BN>
__device__ __forceinline__ void store_tile_output(const f32x16 (&acc)[BM / 64][BN / 64], void* __restrict__ C,
                                                  const TileInfo& ti, int N, int M, int wm, int wn, int frow,
                                                  int half) {
  constexpr int MI = BM / 64, NI = BN / 64;
  const int cols = min(BN, N - ti.col0);
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    const int m = wm * (BM / 2) + mi * 32 + frow;
    if (m >= ti.rows) continue;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = wn * (BN / 2) + ni * 32 + q * 8 + half * 4;
        if (n >= cols) continue;   // (N is a multiple of 8: a group of 4 columns is all in or all out)
        const float v0 = acc[mi][ni][q * 4 + 0], v1 = acc[mi][ni][q * 4 + 1];
        const float v2 = acc[mi][ni][q * 4 + 2], v3 = acc[mi][ni][q * 4 + 3];
        if (MODE == 0) {
          bf16_t* c = static_cast<bf16_t*>(C) + static_cast<int64_t>(ti.row0 + m) * N + ti.col0 + n;
          uint2 p;
          p.x = Elem16<DT>::pack2(v0, v1);
          p.y = Elem16<DT>::pack2(v2, v3);
          *reinterpret_cast<uint2*>(c) = p;
        } else {
          float* c = static_cast<float*>(C) + (static_cast<int64_t>(ti.expert) * M + ti.m0 + m) * N + ti.col0 + n;
          *reinterpret_cast<float4*>(c) = make_float4(v0, v1, v2, v3);
        }
      }
    }
  }
}

// One output tile's products over the k-tiles [kt_begin, kt_end) into `acc`: two LDS stages, the next
// k-tile's loads in flight while the current one is multiplied.  SKIP_DEAD: 32-row blocks past the
// tile's last valid row are not multiplied (their accumulators stay zero).
template <int MODE, int DT, int BM, int BN, bool SKIP_DEAD>
__device__ __forceinline__ void accumulate_tile(const TileInfo& ti, int kt_begin, int kt_end,
                                                f32x16 (&acc)[BM / 64][BN / 64], unsigned char* lds) {
  typedef typename Elem16<DT>::vec8 vec8;
  const Operand opA = ti.opA, opB = ti.opB;
  constexpr bool kAContig = MODE == 0;   // A[r, k]: k contiguous only for the data gradient

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int frow = lane & 31, half = lane >> 5;
  // staging: wavefronts 0, 1 bring in the A tile, 2, 3 the B tile
  const bool stage_b = wave >= 2;
  const int stage_half = wave & 1;
  const int live_rows = ti.rows - wm * (BM / 2);   // valid rows of this wavefront's half of the tile

  constexpr int MI = BM / 64, NI = BN / 64;      // 32 x 32 blocks per wavefront, along m and along n
  constexpr int kATileBytes = BM * kRowBytes;
  constexpr int kStageBytes = (BM + BN) * kRowBytes;
  constexpr int SR = BM > BN ? BM : BN;          // (the staging registers fit the larger operand tile)
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

  u32x4 g[SR / 16];
  auto load = [&](int kt) {
    if (stage_b) load_tile<false, BN>(opB, kt * BK, stage_half, lane, g);
    else load_tile<kAContig, BM>(opA, kt * BK, stage_half, lane, g);
  };
  auto store = [&](unsigned char* buf) {
    if (stage_b) store_tile<false, BN>(buf + kATileBytes, stage_half, lane, g);
    else store_tile<kAContig, BM>(buf, stage_half, lane, g);
  };
  if (kt_end > kt_begin) {
    load(kt_begin);
    store(lds);
  }
  __syncthreads();
  for (int kt = kt_begin; kt < kt_end; ++kt) {
    unsigned char* cur = lds + ((kt - kt_begin) & 1) * kStageBytes;
    unsigned char* nxt = lds + ((kt - kt_begin + 1) & 1) * kStageBytes;
    if (kt + 1 < kt_end) load(kt + 1);
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      vec8 fa[MI], fb[NI];
#pragma unroll
      for (int mi = 0; mi < MI; ++mi)
        fa[mi] = *reinterpret_cast<const vec8*>(cur + lds_chunk(wm * (BM / 2) + mi * 32 + frow, ks * 2 + half));
#pragma unroll
      for (int ni = 0; ni < NI; ++ni)
        fb[ni] = *reinterpret_cast<const vec8*>(cur + kATileBytes + lds_chunk(wn * (BN / 2) + ni * 32 + frow, ks * 2 + half));
#pragma unroll
      for (int mi = 0; mi < MI; ++mi) {
        if (SKIP_DEAD && mi * 32 >= live_rows) continue;   // (uniform over the wavefront)
#pragma unroll
        for (int ni = 0; ni < NI; ++ni)
          acc[mi][ni] = Elem16<DT>::mfma32(fb[ni], fa[mi], acc[mi][ni]);   // D[n][m]: lane = row m, registers = columns n
      }
    }
    if (kt + 1 < kt_end) store(nxt);
    __syncthreads();
  }
}

// MODE 0 (data gradient):   C[r, n]    = sum_k A[r, k] * B[i][k, n]   for the rows r of expert i
//                           A [rows, K] 16-bit, B [n_exp, K, N] 16-bit, C [rows, N] 16-bit
// MODE 1 (weight gradient): C[i][m, n] = sum_{r in expert i} A[r, m] * B[r, n]
//                           A [rows, M] 16-bit, B [rows, N] 16-bit, C [n_exp, M, N] float32
template <int MODE, int DT, int BM, int BN>
__global__ __launch_bounds__(kThreads) void grouped_gemm_bwd_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, void* __restrict__ C,
    const int32_t* __restrict__ offsets, int n_exp, int M, int N, int K) {
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  TileInfo ti;
  if (!locate_tile<MODE, BM, BN>(A, B, offsets, n_exp, M, N, K, ti)) return;
  f32x16 acc[BM / 64][BN / 64];
  accumulate_tile<MODE, DT, BM, BN, false>(ti, 0, ti.kt_count, acc, lds);
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  store_tile_output<MODE, DT, BM, BN>(acc, C, ti, N, M, wave >> 1, wave & 1, lane & 31, lane >> 5);
}

// The split-off tails of the data gradient (see tail_threshold): block (expert, row tile, column tile,
// split) multiplies up to 128 of the expert's tail rows by a 128-column panel over its share of the
// contraction and leaves float32 partial sums in `partial` [splits][n_exp][256][N].
template <int DT>
__global__ __launch_bounds__(kThreads) void grouped_gemm_bwd_tail_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, float* __restrict__ partial,
    const int32_t* __restrict__ offsets, int n_exp, int N, int K, int splits, int tail_cus) {
  constexpr int BM = kTailTile, BN = 128;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  const int tail_thr = tail_threshold(offsets, n_exp, N, tail_cus);
  if (tail_thr == 0) return;
  const int n_tiles = (N + BN - 1) / BN;
  int b = blockIdx.x;
  const int nt = b % n_tiles;
  b /= n_tiles;
  const int split = b % splits;
  b /= splits;
  const int rt = b & 1, expert = b >> 1;
  const int lo = offsets[expert], hi = offsets[expert + 1];
  const int tail = tail_rows_of(hi - lo, tail_thr);
  if (rt * BM >= tail) return;
  TileInfo ti;
  ti.expert = expert;
  ti.row0 = hi - tail + rt * BM;
  ti.rows = min(BM, tail - rt * BM);
  ti.col0 = nt * BN;
  ti.m0 = 0;
  ti.kt_count = (K + BK - 1) / BK;
  ti.opA = Operand{A + static_cast<int64_t>(ti.row0) * K, K, ti.rows, K};
  ti.opB = Operand{B + static_cast<int64_t>(expert) * K * N + ti.col0, N, min(BN, N - ti.col0), K};
  const int per = (ti.kt_count + splits - 1) / splits;
  const int kt_begin = split * per, kt_end = min(ti.kt_count, kt_begin + per);
  f32x16 acc[BM / 64][BN / 64];
  accumulate_tile<0, DT, BM, BN, true>(ti, kt_begin, kt_end, acc, lds);

  // lane: row frow of each 32-row block; register v: column (v / 4) * 8 + half * 4 + v % 4
  const int lane = threadIdx.x & 63, wave = __builtin_amdgcn_readfirstlane(threadIdx.x >> 6);
  const int wm = wave >> 1, wn = wave & 1, frow = lane & 31, half = lane >> 5;
  float* out = partial + ((static_cast<int64_t>(split) * n_exp + expert) * 256 + rt * BM) * N;
  const int cols = min(BN, N - ti.col0);
#pragma unroll
  for (int mi = 0; mi < BM / 64; ++mi) {
    const int m = wm * (BM / 2) + mi * 32 + frow;
    if (m >= ti.rows) continue;
#pragma unroll
    for (int ni = 0; ni < BN / 64; ++ni)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int n = wn * (BN / 2) + ni * 32 + q * 8 + half * 4;
        if (n < cols)
          *reinterpret_cast<float4*>(out + static_cast<int64_t>(m) * N + ti.col0 + n) =
              make_float4(acc[mi][ni][q * 4 + 0], acc[mi][ni][q * 4 + 1], acc[mi][ni][q * 4 + 2], acc[mi][ni][q * 4 + 3]);
      }
  }
}

// Adds the tail kernel's partial sums in split order and stores the tail rows of C [rows, N] (16-bit).
// One block per (expert, tail row), a thread per 8 columns.
template <int DT>
__global__ __launch_bounds__(256) void tail_reduce_kernel(const float* __restrict__ partial, bf16_t* __restrict__ C,
                                                          const int32_t* __restrict__ offsets, int n_exp, int N,
                                                          int splits, int tail_cus) {
  const int tail_thr = tail_threshold(offsets, n_exp, N, tail_cus);
  if (tail_thr == 0) return;
  const int expert = blockIdx.x >> 8, r = blockIdx.x & 255;
  const int lo = offsets[expert], hi = offsets[expert + 1];
  const int tail = tail_rows_of(hi - lo, tail_thr);
  if (r >= tail) return;
  bf16_t* crow = C + static_cast<int64_t>(hi - tail + r) * N;
  for (int n = threadIdx.x * 8; n < N; n += 256 * 8) {   // (N is a multiple of 8)
    float a[8] = {0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f, 0.f};
    for (int sp = 0; sp < splits; ++sp) {
      const float* p = partial + ((static_cast<int64_t>(sp) * n_exp + expert) * 256 + r) * N + n;
      const float4 u = *reinterpret_cast<const float4*>(p), w = *reinterpret_cast<const float4*>(p + 4);
      a[0] += u.x; a[1] += u.y; a[2] += u.z; a[3] += u.w;
      a[4] += w.x; a[5] += w.y; a[6] += w.z; a[7] += w.w;
    }
    u32x4 o;
    o.x = Elem16<DT>::pack2(a[0], a[1]);
    o.y = Elem16<DT>::pack2(a[2], a[3]);
    o.z = Elem16<DT>::pack2(a[4], a[5]);
    o.w = Elem16<DT>::pack2(a[6], a[7]);
    *reinterpret_cast<u32x4*>(crow + n) = o;
  }
}

// The same products on a 256 x 256 x 64 tile with one wavefront per SIMD (256 accumulator registers),
// software-pipelined by hand, because a single wavefront has nobody to hide its latencies behind:
//   * two sets of staging registers: a k-tile is loaded a tile and a half before it is written to LDS
//     (buffer loads whose descriptor ends with the operand's last valid row: tails and phantom tiles
//     read zeros and the loop has no branches); it is written to the other LDS stage during the first
//     two k-steps of an iteration (transposed in registers where the contraction index is the memory
//     row) and the set is reloaded during the last two;
//   * exactly one LDS or memory instruction after each MFMA: a fragment read after the even ones (the
//     fragments of k-step s + 1 are read while the MFMAs of k-step s run), a staging write or load
//     after the odd ones; LDS accesses are inline assembly and every wait is counted by hand (LDS
//     operations complete in order: "lgkmcnt(n)" lets the n youngest stay outstanding);
//   * one barrier per k-tile, after the third k-step: by then every wavefront has written its share
//     of the next stage and read its last fragments of this one; the first fragments of the next
//     tile are read behind it.
// The data gradient needs K to be a multiple of 64 (a k-contiguous operand is not masked along k).
template <int OFF>
__device__ __forceinline__ void lds_read16_at(u32x4& dst, uint32_t addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF) : "memory");
}
template <int OFF>
__device__ __forceinline__ void lds_write16_at(uint32_t addr, const u32x4& v) {
  asm volatile("ds_write_b128 %0, %1 offset:%2" : : "v"(addr), "v"(v), "n"(OFF) : "memory");
}
#define PPMOE_BWD_TIE8(f) \
  "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7])

template <int MODE, int DT>
__global__ __launch_bounds__(kThreads) void grouped_gemm_bwd_pipelined_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, void* __restrict__ C,
    const int32_t* __restrict__ offsets, int n_exp, int M, int N, int K, int tail_cus) {
  constexpr int BM = 256, BN = 256, MI = 4, NI = 4;
  constexpr int kATileBytes = BM * kRowBytes;
  constexpr int kStageBytes = (BM + BN) * kRowBytes;
  extern __shared__ __attribute__((aligned(16))) unsigned char lds[];
  typedef typename Elem16<DT>::vec8 vec8;

  TileInfo ti;
  if (!locate_tile<MODE, BM, BN>(A, B, offsets, n_exp, M, N, K, ti, MODE == 0 ? tail_cus : 0)) return;
  const int kt_count = ti.kt_count;

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const int frow = lane & 31, half = lane >> 5;
  const bool stage_b = wave >= 2;          // wavefronts 0, 1 bring in the A tile, 2, 3 the B tile
  const int stage_half = wave & 1;
  const Operand op = stage_b ? ti.opB : ti.opA;
  const int col_start = stage_b ? ti.col0 : ti.m0;   // (row-contiguous operands: first column of the tile)
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
      (const __attribute__((address_space(3))) unsigned char*)lds));

  f32x16 acc[MI][NI];
#pragma unroll
  for (int mi = 0; mi < MI; ++mi)
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

  // Fragment addresses: row r, 16-byte chunk 2 ks + half, swizzled with (r >> 4) & 7 = 2 i + b for
  // the i-th 32-row block (b = frow >> 4): chunk 2 (ks ^ i) + (half ^ b), i.e. a per-lane base plus
  // the constant i * 32 rows + (ks ^ i) * 32 bytes.
  const int b4 = frow >> 4;
  const uint32_t fa_addr = lds0 + (wm * 128 + frow) * kRowBytes + ((half ^ b4) << 4);
  const uint32_t fb_addr = lds0 + kATileBytes + (wn * 128 + frow) * kRowBytes + ((half ^ b4) << 4);

// One MFMA, pinned where it is written (the scheduler may not move anything across it).
#define PPMOE_BWD_MFMA(f, mi, ni)                                                   \
  do {                                                                              \
    __builtin_amdgcn_sched_barrier(0);                                              \
    acc[mi][ni] = Elem16<DT>::mfma32(__builtin_bit_cast(vec8, f[4 + ni]), __builtin_bit_cast(vec8, f[mi]), acc[mi][ni]); \
    __builtin_amdgcn_sched_barrier(0);                                              \
  } while (0)
#define PPMOE_BWD_WAIT(n, f) asm volatile("s_waitcnt lgkmcnt(" #n ")" : PPMOE_BWD_TIE8(f) : : "memory")
// fragment i of the A / B tile for k-step NKS, from the stage whose fragment base addresses are fa / fb
#define PPMOE_BWD_RA(f, i, NKS, fa) lds_read16_at<(i) * 32 * kRowBytes + (((NKS) ^ (i)) << 5)>(f[i], fa)
#define PPMOE_BWD_RB(f, i, NKS, fb) lds_read16_at<(i) * 32 * kRowBytes + (((NKS) ^ (i)) << 5)>(f[4 + (i)], fb)
// One k-step: 16 MFMAs on `cur`; after the even ones the eight fragment reads of k-step NKS into `nxt`
// (order A0 B0 B1 A1 B2 B3 A2 A3, the order in which the MFMAs of the next k-step first need them:
// MFMAs 0, 0, 1, 2, 4, 5, 8, 10); after the odd ones ODD(0..7).  W0..W10: how many LDS operations
// may still be outstanding when MFMA 0, 1, 2, 4, 5, 8, 10 issues (-1: nothing to wait for).
#define PPMOE_BWD_STEP(cur, nxt, NKS, fa, fb, W0, W1, W2, W4, W5, W8, W10, ODD) \
  do {                                                                         \
    W0(cur);  PPMOE_BWD_MFMA(cur, 0, 0); PPMOE_BWD_RA(nxt, 0, NKS, fa);         \
    W1(cur);  PPMOE_BWD_MFMA(cur, 0, 1); ODD(0);                                \
    W2(cur);  PPMOE_BWD_MFMA(cur, 1, 0); PPMOE_BWD_RB(nxt, 0, NKS, fb);         \
              PPMOE_BWD_MFMA(cur, 1, 1); ODD(1);                                \
    W4(cur);  PPMOE_BWD_MFMA(cur, 0, 2); PPMOE_BWD_RB(nxt, 1, NKS, fb);         \
    W5(cur);  PPMOE_BWD_MFMA(cur, 0, 3); ODD(2);                                \
              PPMOE_BWD_MFMA(cur, 1, 2); PPMOE_BWD_RA(nxt, 1, NKS, fa);         \
              PPMOE_BWD_MFMA(cur, 1, 3); ODD(3);                                \
    W8(cur);  PPMOE_BWD_MFMA(cur, 2, 0); PPMOE_BWD_RB(nxt, 2, NKS, fb);         \
              PPMOE_BWD_MFMA(cur, 2, 1); ODD(4);                                \
    W10(cur); PPMOE_BWD_MFMA(cur, 3, 0); PPMOE_BWD_RB(nxt, 3, NKS, fb);         \
              PPMOE_BWD_MFMA(cur, 3, 1); ODD(5);                                \
              PPMOE_BWD_MFMA(cur, 2, 2); PPMOE_BWD_RA(nxt, 2, NKS, fa);         \
              PPMOE_BWD_MFMA(cur, 2, 3); ODD(6);                                \
              PPMOE_BWD_MFMA(cur, 3, 2); PPMOE_BWD_RA(nxt, 3, NKS, fa);         \
              PPMOE_BWD_MFMA(cur, 3, 3); ODD(7);                                \
  } while (0)
#define PPMOE_BWD_NOWAIT(f) do { } while (0)
#define PPMOE_BWD_WAIT6(f) PPMOE_BWD_WAIT(6, f)
#define PPMOE_BWD_WAIT7(f) PPMOE_BWD_WAIT(7, f)
#define PPMOE_BWD_WAIT8(f) PPMOE_BWD_WAIT(8, f)
#define PPMOE_BWD_WAIT9(f) PPMOE_BWD_WAIT(9, f)
#define PPMOE_BWD_WAIT10(f) PPMOE_BWD_WAIT(10, f)
#define PPMOE_BWD_WAIT11(f) PPMOE_BWD_WAIT(11, f)
#define PPMOE_BWD_WAIT12(f) PPMOE_BWD_WAIT(12, f)
#define PPMOE_BWD_WAIT13(f) PPMOE_BWD_WAIT(13, f)

  auto k_loop = [&](auto contig_c) __attribute__((always_inline)) {
    constexpr bool CONTIG = decltype(contig_c)::value;
    u32x4 g0[16], g1[16];   // staging set 0: even k-tiles, set 1: odd k-tiles
    // this lane's byte offset inside a k-tile of its operand, and where it writes in an LDS stage
    const uint32_t ld2 = static_cast<uint32_t>(op.ld) * 2u;
    uint32_t loff, st_addr;
    const int ch = lane & 7;
    if (CONTIG) {
      const int lrow = (lane >> 3) + 8 * stage_half;
      loff = lrow * ld2 + ch * 16;
      st_addr = lds0 + lrow * kRowBytes;
    } else {
      const int rg = lane & 15, kg = stage_half * 4 + (lane >> 4);
      loff = kg * 8 * ld2 + rg * 16;
      st_addr = lds0 + (stage_b ? kATileBytes : 0) + rg * 8 * kRowBytes + ((kg ^ (rg >> 1)) << 4);   // rows g * 128 + rg * 8 + r: (row >> 4) & 7 = rg >> 1
    }
    // Extent of the operand from the first element of k-tile 0 to the end of its last valid row, and
    // how much of it a step along k leaves behind: the descriptor of k-tile kt covers what is left,
    // and nothing at all for a phantom tile (kt >= kt_count): zeros, no memory touched.
    const int64_t extent0 = CONTIG ? (static_cast<int64_t>(op.rows - 1) * op.ld + op.ks) * 2
                                   : (static_cast<int64_t>(op.ks) * op.ld - col_start) * 2;
    const int64_t k_step = CONTIG ? BK * 2 : static_cast<int64_t>(BK) * ld2;
    auto gload = [&](u32x4 (&g)[16], int kt, int i) __attribute__((always_inline)) {
      const unsigned char* base = reinterpret_cast<const unsigned char*>(op.base) + kt * k_step;
      int64_t bytes = extent0 - kt * k_step;
      bytes = (bytes < 0 || kt >= kt_count) ? 0 : bytes;
      const int records = static_cast<int>(bytes < 0x7fffffff ? bytes : 0x7fffffff);
      const __amdgpu_buffer_rsrc_t rsrc =
          __builtin_amdgcn_make_buffer_rsrc(const_cast<unsigned char*>(base), 0, records, 0x00020000);
      // CONTIG: rows lrow + 16 i.  Otherwise i = gq * 8 + kk: memory row kg * 8 + kk, columns gq * 128 + rg * 8
      const uint32_t so = CONTIG ? i * 16 * ld2 : (i & 7) * ld2 + (i >> 3) * 256;
      g[i] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, loff, so, 0);
    };
    // the i-th of the 16 LDS writes of a staged tile into the stage at byte offset `stage`
    auto gstore = [&](const u32x4 (&g)[16], uint32_t stage, auto i_c) __attribute__((always_inline)) {
      constexpr int i = decltype(i_c)::value;
      if (CONTIG) {
        lds_write16_at<i * 16 * kRowBytes>(st_addr + stage + ((ch ^ (i & 7)) << 4), g[i]);
      } else {
        // g[gq * 8 + kk] dword q holds tile rows 2q (low half) and 2q + 1 (high half) at k = kk; the
        // chunk of tile row r wants, in dword q, k = 2q (low) and 2q + 1 (high).
        constexpr int gq = i >> 3, r = i & 7;
        constexpr uint32_t sel = (r & 1) ? 0x07060302u : 0x05040100u;
        u32x4 o;
        o.x = __builtin_amdgcn_perm(g[gq * 8 + 1][r >> 1], g[gq * 8 + 0][r >> 1], sel);
        o.y = __builtin_amdgcn_perm(g[gq * 8 + 3][r >> 1], g[gq * 8 + 2][r >> 1], sel);
        o.z = __builtin_amdgcn_perm(g[gq * 8 + 5][r >> 1], g[gq * 8 + 4][r >> 1], sel);
        o.w = __builtin_amdgcn_perm(g[gq * 8 + 7][r >> 1], g[gq * 8 + 6][r >> 1], sel);
        lds_write16_at<(gq * 128 + r) * kRowBytes>(st_addr + stage, o);
      }
    };
#define PPMOE_BWD_IC(i) std::integral_constant<int, (i)>{}

    // ---- prologue: tile 0 through set 0 into stage 0; tiles 1 and 2 in flight in sets 1 and 0 -----
#pragma unroll
    for (int i = 0; i < 16; ++i) gload(g0, 0, i);
    gstore(g0, 0, PPMOE_BWD_IC(0)); gstore(g0, 0, PPMOE_BWD_IC(1)); gstore(g0, 0, PPMOE_BWD_IC(2)); gstore(g0, 0, PPMOE_BWD_IC(3));
    gstore(g0, 0, PPMOE_BWD_IC(4)); gstore(g0, 0, PPMOE_BWD_IC(5)); gstore(g0, 0, PPMOE_BWD_IC(6)); gstore(g0, 0, PPMOE_BWD_IC(7));
    gstore(g0, 0, PPMOE_BWD_IC(8)); gstore(g0, 0, PPMOE_BWD_IC(9)); gstore(g0, 0, PPMOE_BWD_IC(10)); gstore(g0, 0, PPMOE_BWD_IC(11));
    gstore(g0, 0, PPMOE_BWD_IC(12)); gstore(g0, 0, PPMOE_BWD_IC(13)); gstore(g0, 0, PPMOE_BWD_IC(14)); gstore(g0, 0, PPMOE_BWD_IC(15));
#pragma unroll
    for (int i = 0; i < 16; ++i) gload(g1, 1, i);
#pragma unroll
    for (int i = 0; i < 16; ++i) gload(g0, 2, i);
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    __builtin_amdgcn_s_barrier();
    asm volatile("" ::: "memory");
    u32x4 f0[8], f1[8];
    const uint32_t fa0 = fa_addr, fb0 = fb_addr, fa1 = fa_addr + kStageBytes, fb1 = fb_addr + kStageBytes;
    PPMOE_BWD_RA(f0, 0, 0, fa0); PPMOE_BWD_RB(f0, 0, 0, fb0); PPMOE_BWD_RB(f0, 1, 0, fb0); PPMOE_BWD_RA(f0, 1, 0, fa0);
    PPMOE_BWD_RB(f0, 2, 0, fb0); PPMOE_BWD_RB(f0, 3, 0, fb0); PPMOE_BWD_RA(f0, 2, 0, fa0); PPMOE_BWD_RA(f0, 3, 0, fa0);

    // One iteration: k-tile kt out of the stage at `fa_c / fb_c`, the staged tile kt + 1 (set G) into
    // the stage at byte offset ST_N (fragment addresses fa_n / fb_n), then tile kt + 3 into set G.
    // Waits: LDS operations issued after fragment read i of a k-step with writes: 15 - 2 i, without:
    // 7 - i; issued in the current k-step before MFMA j: j with writes, (j + 1) / 2 without.
#define PPMOE_BWD_ITER(kt, G, fa_c, fb_c, fa_n, fb_n, ST_N)                                                    \
  do {                                                                                                         \
    PPMOE_BWD_STEP(f0, f1, 1, fa_c, fb_c, PPMOE_BWD_WAIT6, PPMOE_BWD_WAIT6, PPMOE_BWD_WAIT6, PPMOE_BWD_WAIT7,  \
                   PPMOE_BWD_WAIT7, PPMOE_BWD_WAIT9, PPMOE_BWD_WAIT10, PPMOE_BWD_ODD_W0);                      \
    PPMOE_BWD_STEP(f1, f0, 2, fa_c, fb_c, PPMOE_BWD_WAIT13, PPMOE_BWD_WAIT12, PPMOE_BWD_WAIT11, PPMOE_BWD_WAIT11, \
                   PPMOE_BWD_WAIT10, PPMOE_BWD_WAIT11, PPMOE_BWD_WAIT11, PPMOE_BWD_ODD_W1);                    \
    PPMOE_BWD_STEP(f0, f1, 3, fa_c, fb_c, PPMOE_BWD_WAIT13, PPMOE_BWD_WAIT12, PPMOE_BWD_WAIT10, PPMOE_BWD_WAIT9, \
                   PPMOE_BWD_WAIT8, PPMOE_BWD_WAIT7, PPMOE_BWD_WAIT6, PPMOE_BWD_ODD_G0);                       \
    asm volatile("s_waitcnt lgkmcnt(0)" : PPMOE_BWD_TIE8(f1) : : "memory");                                    \
    __builtin_amdgcn_s_barrier();                                                                              \
    asm volatile("" ::: "memory");                                                                             \
    PPMOE_BWD_STEP(f1, f0, 0, fa_n, fb_n, PPMOE_BWD_NOWAIT, PPMOE_BWD_NOWAIT, PPMOE_BWD_NOWAIT, PPMOE_BWD_NOWAIT, \
                   PPMOE_BWD_NOWAIT, PPMOE_BWD_NOWAIT, PPMOE_BWD_NOWAIT, PPMOE_BWD_ODD_G1);                    \
  } while (0)

    for (int kt = 0; kt < kt_count; kt += 2) {
#define PPMOE_BWD_ODD_W0(i) gstore(g1, kStageBytes, PPMOE_BWD_IC(i))
#define PPMOE_BWD_ODD_W1(i) gstore(g1, kStageBytes, PPMOE_BWD_IC(8 + (i)))
#define PPMOE_BWD_ODD_G0(i) gload(g1, kt + 3, i)
#define PPMOE_BWD_ODD_G1(i) gload(g1, kt + 3, 8 + (i))
      PPMOE_BWD_ITER(kt, g1, fa0, fb0, fa1, fb1, kStageBytes);
#undef PPMOE_BWD_ODD_W0
#undef PPMOE_BWD_ODD_W1
#undef PPMOE_BWD_ODD_G0
#undef PPMOE_BWD_ODD_G1
#define PPMOE_BWD_ODD_W0(i) gstore(g0, 0, PPMOE_BWD_IC(i))
#define PPMOE_BWD_ODD_W1(i) gstore(g0, 0, PPMOE_BWD_IC(8 + (i)))
#define PPMOE_BWD_ODD_G0(i) gload(g0, kt + 4, i)
#define PPMOE_BWD_ODD_G1(i) gload(g0, kt + 4, 8 + (i))
      PPMOE_BWD_ITER(kt + 1, g0, fa1, fb1, fa0, fb0, 0);
#undef PPMOE_BWD_ODD_W0
#undef PPMOE_BWD_ODD_W1
#undef PPMOE_BWD_ODD_G0
#undef PPMOE_BWD_ODD_G1
    }
    // (the fragments read behind the last barrier are not used; let them land before the registers die)
    asm volatile("s_waitcnt lgkmcnt(0)" : PPMOE_BWD_TIE8(f0) : : "memory");
  };
  if (MODE == 0 && !stage_b) k_loop(std::true_type{});
  else k_loop(std::false_type{});
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");

  // Epilogue through LDS, 64 tile rows (32 of each half of the tile) per pass: the accumulators
  // (a lane has one row and groups of four columns) are written into a [64][row] buffer and read back
  // as 16-byte pieces of whole rows, the four wavefronts on neighbouring rows, so that a store
  // instruction covers one or two contiguous tile rows (a kilobyte) instead of 16 or 32 bytes of each
  // of 32 rows (alone, that pattern writes at about a third of the rate of whole rows).  Two buffers
  // alternate: one barrier per pass.
  __syncthreads();   // every wavefront has read its last fragments: the stages are free
  constexpr int EB = MODE == 1 ? 4 : 2;            // bytes per output element
  constexpr int kOutRowB = BN * EB;                // one tile row
  constexpr int kOutPitch = kOutRowB + 16;
  constexpr int kOutBuf = 64 * kOutPitch;
  constexpr int LPR = kOutRowB / 16, RPI = 64 / LPR;   // lanes per row, rows per instruction
  static_assert(2 * kOutBuf <= lds_bytes(BM, BN), "the two output buffers fit in the stages");
  unsigned char* outb = static_cast<unsigned char*>(C) +
      (MODE == 1 ? ((static_cast<int64_t>(ti.expert) * M + ti.m0) * N + ti.col0) * 4
                 : (static_cast<int64_t>(ti.row0) * N + ti.col0) * 2);
  const int64_t out_pitch = static_cast<int64_t>(N) * EB;
  const int cols_b = min(BN, N - ti.col0) * EB;    // valid bytes of a tile row (N is a multiple of 8)
#pragma unroll
  for (int mi = 0; mi < MI; ++mi) {
    unsigned char* buf = lds + (mi & 1) * kOutBuf;
    unsigned char* wrow = buf + (wm * 32 + frow) * kOutPitch;
#pragma unroll
    for (int ni = 0; ni < NI; ++ni)
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        const int col = wn * 128 + ni * 32 + q * 8 + half * 4;
        const float v0 = acc[mi][ni][q * 4 + 0], v1 = acc[mi][ni][q * 4 + 1];
        const float v2 = acc[mi][ni][q * 4 + 2], v3 = acc[mi][ni][q * 4 + 3];
        if (MODE == 1) {
          *reinterpret_cast<float4*>(wrow + col * 4) = make_float4(v0, v1, v2, v3);
        } else {
          uint2 p;
          p.x = Elem16<DT>::pack2(v0, v1);
          p.y = Elem16<DT>::pack2(v2, v3);
          *reinterpret_cast<uint2*>(wrow + col * 2) = p;
        }
      }
    __syncthreads();
#pragma unroll
    for (int i = 0; i < 16 / RPI; ++i) {
      const int lr = (i * 4 + wave) * RPI + lane / LPR;          // row of the buffer
      const int cb = (lane % LPR) * 16;                          // byte offset in the row
      const int m = (lr < 32 ? lr : 128 - 32 + lr) + mi * 32;    // row of the tile
      if (m < ti.rows && cb < cols_b)
        *reinterpret_cast<u32x4*>(outb + m * out_pitch + cb) = *reinterpret_cast<const u32x4*>(buf + lr * kOutPitch + cb);
    }
  }
}
#undef PPMOE_BWD_ITER
#undef PPMOE_BWD_IC
#undef PPMOE_BWD_STEP
#undef PPMOE_BWD_RA
#undef PPMOE_BWD_RB
#undef PPMOE_BWD_WAIT
#undef PPMOE_BWD_MFMA

// H = GeLU(U) (not stored when H is NULL: the caller has it) and dU = dH * GeLU'(U) over the packed
// rows [0, offsets[n_exp]) x F, one row per block
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
      if (H != nullptr) reinterpret_cast<u32x4*>(H)[at] = u32x4{hw[0], hw[1], hw[2], hw[3]};   // (uniform)
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

// H = GeLU(U) alone, the same arithmetic.
template <int DT>
__global__ __launch_bounds__(256) void gelu_rows_kernel(const bf16_t* __restrict__ U, bf16_t* __restrict__ H,
                                                        const int32_t* __restrict__ offsets, int n_exp, int F) {
  const int64_t pieces = static_cast<int64_t>(offsets[n_exp]) * (F / 8);   // 16-byte pieces
  for (int64_t at = static_cast<int64_t>(blockIdx.x) * 256 + threadIdx.x; at < pieces;
       at += static_cast<int64_t>(gridDim.x) * 256) {
    const u32x4 u4 = reinterpret_cast<const u32x4*>(U)[at];
    const uint32_t uw[4] = {u4.x, u4.y, u4.z, u4.w};
    uint32_t hw[4];
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      float u[2], h[2];
      Elem16<DT>::widen2(uw[j], u[0], u[1]);
#pragma unroll
      for (int e = 0; e < 2; ++e) {
        const float z2 = 1.5957691216057308f * u[e] * fmaf(0.044715f * u[e], u[e], 1.0f);
        h[e] = u[e] * (1.0f / (1.0f + __expf(-z2)));
      }
      hw[j] = Elem16<DT>::pack2(h[0], h[1]);
    }
    reinterpret_cast<u32x4*>(H)[at] = u32x4{hw[0], hw[1], hw[2], hw[3]};
  }
}

}  // namespace bwd

hipError_t launch_gelu_rows(const moe_config& c, const void* U, void* H, const int32_t* offsets, int64_t rows,
                            hipStream_t s) {
  if (rows <= 0) return hipSuccess;
  const int64_t pieces = rows * (c.F / 8);
  const int blocks = static_cast<int>(pieces / 256 < 256 * 16 ? (pieces + 255) / 256 : 256 * 16);
  if (c.in_dtype == MOE_F16)
    bwd::gelu_rows_kernel<MOE_F16><<<blocks, 256, 0, s>>>(static_cast<const bf16_t*>(U), static_cast<bf16_t*>(H),
                                                          offsets, c.local_count, c.F);
  else
    bwd::gelu_rows_kernel<MOE_BF16><<<blocks, 256, 0, s>>>(static_cast<const bf16_t*>(U), static_cast<bf16_t*>(H),
                                                           offsets, c.local_count, c.F);
  return hipGetLastError();
}

// Partial sums of the split-off tails of dX: [splits][local experts][256][d] float32 (no tail
// launches with more than 16 local experts: the buffer would grow past what the launches can save).
static size_t tail_partial_bytes(const moe_config& c) {
  if (c.local_count > 16) return 0;
  return static_cast<size_t>(bwd::kTailSplitsMax) * c.local_count * 256 * c.d * sizeof(float);
}

// Compute units of the current device (asked once per device: the launcher may run under stream capture).
static int cus_of_current_device() {
  static std::atomic<int> cached[64];
  int dev = 0;
  if (hipGetDevice(&dev) != hipSuccess || dev < 0 || dev >= 64) return 256;
  int cus = cached[dev].load(std::memory_order_relaxed);
  if (cus == 0) {
    if (hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || cus <= 0) cus = 256;
    cached[dev].store(cus, std::memory_order_relaxed);
  }
  return cus;
}

size_t expert_ffn_backward_scratch_bytes(const moe_config& c, int64_t rows) {
  // U, H, dU: three [rows, F] 16-bit buffers (256-byte aligned), the forward GEMM's scratch, the
  // partial sums of dX's tails
  const size_t one = (static_cast<size_t>(rows) * c.F * 2 + 255) & ~size_t(255);
  return 3 * one + ((grouped_gemm_workspace_bytes() + 255) & ~size_t(255)) + tail_partial_bytes(c);
}

hipError_t launch_expert_ffn_backward(const moe_config& c, int64_t rows, const void* x_sliced,
                                      const int32_t* offsets, const void* W1, const void* W2,
                                      const void* dY, void* dX, float* dW1, float* dW2, void* scratch,
                                      hipStream_t s, float* row_dot, const void* U_saved, const void* H_saved) {
  using namespace bwd;
  // (rows == 0: no packed row can exist; every launch below is then empty except the two weight
  // gradients, whose tiles store zeros)
  const size_t one = (static_cast<size_t>(rows) * c.F * 2 + 255) & ~size_t(255);
  unsigned char* ws = static_cast<unsigned char*>(scratch);
  const bool saved = U_saved != nullptr && H_saved != nullptr;
  const bf16_t* U = saved ? static_cast<const bf16_t*>(U_saved) : reinterpret_cast<const bf16_t*>(ws);
  const bf16_t* H = saved ? static_cast<const bf16_t*>(H_saved) : reinterpret_cast<const bf16_t*>(ws + one);
  bf16_t* H_out = saved ? nullptr : reinterpret_cast<bf16_t*>(ws + one);
  bf16_t* dU = reinterpret_cast<bf16_t*>(ws + 2 * one);
  void* gemm_ws = ws + 3 * one;
  float* tail_partial = reinterpret_cast<float*>(ws + 3 * one + ((grouped_gemm_workspace_bytes() + 255) & ~size_t(255)));
  const int N = c.local_count;
  const bf16_t* xs = static_cast<const bf16_t*>(x_sliced);
  const bf16_t* w1 = static_cast<const bf16_t*>(W1);
  const bf16_t* w2 = static_cast<const bf16_t*>(W2);
  const bf16_t* dy = static_cast<const bf16_t*>(dY);

  // U = X A (the forward's first GEMM without its activation), unless the forward kept it
  if (!saved) {
    hipError_t e = launch_grouped_gemm(c.in_dtype, false, x_sliced, W1, ws, offsets, N, rows, c.F, c.d, gemm_ws, s);
    if (e != hipSuccess) return e;
  }

  // Tile shape per launch: the pipelined 256 x 256 kernel (one block per CU, half the LDS and L2
  // traffic per flop, latencies hidden by its schedule) unless that leaves more than half of the CUs
  // without a tile; then 128 x 128 (two blocks per CU, compiler-scheduled; also K not a multiple of
  // 64).  The host knows the row count only as a bound (the counts live on the device).
  const int n_cus = cus_of_current_device();
  static std::atomic<uint64_t> attrs_done{0};
  const hipError_t attrs = once_per_device(attrs_done, [] {
    const void* small[] = {reinterpret_cast<const void*>(grouped_gemm_bwd_kernel<0, MOE_BF16, 128, 128>),
                           reinterpret_cast<const void*>(grouped_gemm_bwd_kernel<1, MOE_BF16, 128, 128>),
                           reinterpret_cast<const void*>(grouped_gemm_bwd_kernel<0, MOE_F16, 128, 128>),
                           reinterpret_cast<const void*>(grouped_gemm_bwd_kernel<1, MOE_F16, 128, 128>)};
    const void* big[] = {reinterpret_cast<const void*>(grouped_gemm_bwd_pipelined_kernel<0, MOE_BF16>),
                         reinterpret_cast<const void*>(grouped_gemm_bwd_pipelined_kernel<1, MOE_BF16>),
                         reinterpret_cast<const void*>(grouped_gemm_bwd_pipelined_kernel<0, MOE_F16>),
                         reinterpret_cast<const void*>(grouped_gemm_bwd_pipelined_kernel<1, MOE_F16>)};
    for (const void* k : small) {
      hipError_t err = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(128, 128));
      if (err != hipSuccess) return err;
    }
    for (const void* k : big) {
      hipError_t err = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(256, 256));
      if (err != hipSuccess) return err;
    }
    const void* tail[] = {reinterpret_cast<const void*>(grouped_gemm_bwd_tail_kernel<MOE_BF16>),
                          reinterpret_cast<const void*>(grouped_gemm_bwd_tail_kernel<MOE_F16>)};
    for (const void* k : tail) {
      hipError_t err = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, lds_bytes(kTailTile, 128));
      if (err != hipSuccess) return err;
    }
    return hipSuccess;
  });
  if (attrs != hipSuccess) return attrs;
  // MODE 0: m_out = the packed rows (their tiles per expert: at most rows / BM + N in all); MODE 1:
  // m_out x n_out is one expert's weight matrix.
  auto tiles_of = [&](int mode, int64_t m_out, int n_out, int bm, int bn) -> int64_t {
    const int64_t nt = (n_out + bn - 1) / bn;
    return mode == 0 ? ((m_out + bm - 1) / bm + N) * nt : static_cast<int64_t>(N) * ((m_out + bm - 1) / bm) * nt;
  };
#define PPMOE_BWD(MODE, a, b, cc, m, n, k, m_out, tail_cus)                                                    \
  do {                                                                                                         \
    const bool big = 2 * tiles_of(MODE, m_out, n, 256, 256) >= n_cus && (MODE == 1 || (k) % BK == 0);          \
    const int t = big ? 256 : 128;                                                                             \
    const unsigned grid = static_cast<unsigned>((tiles_of(MODE, m_out, n, t, t) + 7) / 8 * 8);                 \
    const size_t shm = lds_bytes(t, t);                                                                        \
    if (big && c.in_dtype == MOE_F16)                                                                          \
      grouped_gemm_bwd_pipelined_kernel<MODE, MOE_F16><<<grid, kThreads, shm, s>>>(a, b, cc, offsets, N, m, n, k, tail_cus); \
    else if (big)                                                                                              \
      grouped_gemm_bwd_pipelined_kernel<MODE, MOE_BF16><<<grid, kThreads, shm, s>>>(a, b, cc, offsets, N, m, n, k, tail_cus); \
    else if (c.in_dtype == MOE_F16)                                                                            \
      grouped_gemm_bwd_kernel<MODE, MOE_F16, 128, 128><<<grid, kThreads, shm, s>>>(a, b, cc, offsets, N, m, n, k);       \
    else                                                                                                       \
      grouped_gemm_bwd_kernel<MODE, MOE_BF16, 128, 128><<<grid, kThreads, shm, s>>>(a, b, cc, offsets, N, m, n, k);      \
  } while (0)

  // dH = dY B^T  (into the dU buffer), then H = GeLU(U), dU = dH * GeLU'(U) in place
  PPMOE_BWD(0, dy, w2, dU, 0, c.F, c.d, rows, 0);
  {
    const int blocks = static_cast<int>(rows < 256 * 16 ? (rows > 0 ? rows : 1) : 256 * 16);
    if (c.in_dtype == MOE_F16)
      act_backward_kernel<MOE_F16><<<blocks, 256, 0, s>>>(U, dU, H_out, dU, row_dot, offsets, N, c.F);
    else
      act_backward_kernel<MOE_BF16><<<blocks, 256, 0, s>>>(U, dU, H_out, dU, row_dot, offsets, N, c.F);
  }
  // dX = dU A^T; with a long contraction the 256 x 256 launch may leave the experts' tail rows to two
  // small launches of their own (every block of the three takes that decision from the row counts)
  const bool dx_big = 2 * tiles_of(0, rows, c.d, 256, 256) >= n_cus && c.F % BK == 0;
  const int tail_cus = (dx_big && c.F >= 4096 && tail_partial_bytes(c) > 0) ? n_cus : 0;
  PPMOE_BWD(0, dU, w1, dX, 0, c.d, c.F, rows, tail_cus);
  if (tail_cus > 0) {
    int splits = c.F / BK / 16;
    splits = splits < 1 ? 1 : splits > kTailSplitsMax ? kTailSplitsMax : splits;
    const unsigned tail_grid = static_cast<unsigned>(N * 2 * ((c.d + 127) / 128) * splits);
    if (c.in_dtype == MOE_F16) {
      grouped_gemm_bwd_tail_kernel<MOE_F16><<<tail_grid, kThreads, lds_bytes(kTailTile, 128), s>>>(
          dU, w1, tail_partial, offsets, N, c.d, c.F, splits, tail_cus);
      tail_reduce_kernel<MOE_F16><<<N * 256, 256, 0, s>>>(tail_partial, static_cast<bf16_t*>(dX), offsets, N,
                                                                c.d, splits, tail_cus);
    } else {
      grouped_gemm_bwd_tail_kernel<MOE_BF16><<<tail_grid, kThreads, lds_bytes(kTailTile, 128), s>>>(
          dU, w1, tail_partial, offsets, N, c.d, c.F, splits, tail_cus);
      tail_reduce_kernel<MOE_BF16><<<N * 256, 256, 0, s>>>(tail_partial, static_cast<bf16_t*>(dX), offsets, N,
                                                                 c.d, splits, tail_cus);
    }
  }
  // dB^T[i] = dY_i^T H_i  ([d, F]);  dA^T[i] = dU_i^T X_i  ([F, d])
  PPMOE_BWD(1, dy, H, dW2, c.d, c.F, 0, c.d, 0);
  PPMOE_BWD(1, dU, xs, dW1, c.F, c.d, 0, c.F, 0);
#undef PPMOE_BWD
  return hipGetLastError();
}

}  // namespace ppmoe
