// Fast path of the grouped expert GEMMs (Section 3.3.2; FFN = GeLU(X A) B, Section 3.1.3) for bf16
// with K a multiple of 64:
//
//   C[r, n] = act( sum_k A[r, k] * B[i][n, k] ),  offsets[i] <= r < offsets[i+1]
//
// Block tile 256 x 256 x 64, four wavefronts (one per SIMD), each owning a 128 x 128 sub-tile as
// 4 x 4 MFMA 32x32x16 bf16 accumulators (256 accumulator registers).
//
// What bounds this kernel is the L2 -> CU fetch path (a 256x256 tile needs 32 bytes per CU per clock
// at full MFMA rate), so the loop is built around keeping that path evenly busy:
//   * global loads are 16 bytes per lane, 8 lanes per row: every request is a whole 128-byte line;
//   * loads are issued four at a time between MFMAs, all through the K loop, never in a burst;
//   * a load stays in flight in registers for a whole tile time (64 MFMAs) before it is written to
//     LDS, and LDS holds two tiles (written one tile ahead of use): three tiles deep in total;
//   * one barrier per tile, placed after the third of the four k-steps, when every wavefront has
//     already fetched the last fragments of the current tile: the fragments of the next tile are
//     prefetched behind it, so no LDS latency is exposed at the tile boundary.
//
// LDS layout of a tile buffer: 256 token rows then 256 weight rows of 128 bytes (eight 16-byte
// pieces); piece p of row r sits at slot p ^ ((r >> 1) & 7).  A ds_read_b128 serves 16 lanes per
// cycle (16 consecutive rows, same logical piece) from 64 banks, and with this swizzle they touch 16
// different 16-byte slots; so do the 16 lanes (2 rows x 8 pieces) of a ds_write_b128.
//
// All LDS traffic is inline assembly with hand-counted lgkmcnt waits, so that the MFMA stream never
// waits for more than it needs; global loads are plain loads (the compiler counts vmcnt for them).

#include "common.h"

namespace ppmoe {

typedef __attribute__((__vector_size__(8 * sizeof(__bf16)))) __bf16 bf16x8;
typedef __attribute__((__vector_size__(16 * sizeof(float)))) float f32x16;

namespace fast {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kThreads = 256;
constexpr int kOperandBytes = BM * BK * 2;     // 32 KiB
constexpr int kBufBytes = 2 * kOperandBytes;   // 64 KiB: one tile (tokens + weights)
constexpr int kLdsBytes = 2 * kBufBytes;       // 128 KiB

__device__ __forceinline__ float gelu_tanh(float u) {
  // 0.5 u (1 + tanh(z)) = u / (1 + exp(-2 z)),  z = sqrt(2/pi) (u + 0.044715 u^3)
  // exp and the reciprocal are single hardware instructions (about 1 ulp each), ample for a bf16 result.
  const float z2 = -2.302208198f * u * fmaf(0.044715f * u, u, 1.0f);   // -2 sqrt(2/pi) log2(e) (u + 0.044715 u^3)
  return u * __builtin_amdgcn_rcpf(1.0f + __builtin_amdgcn_exp2f(z2));
}

template <int OFF>
__device__ __forceinline__ void lds_read16(bf16x8& dst, uint32_t addr) {
  asm volatile("ds_read_b128 %0, %1 offset:%2" : "=v"(dst) : "v"(addr), "n"(OFF) : "memory");
}
template <int OFF>
__device__ __forceinline__ void lds_write16(uint32_t addr, const u32x4& v) {
  asm volatile("ds_write_b128 %0, %1 offset:%2" : : "v"(addr), "v"(v), "n"(OFF) : "memory");
}

#define PPMOE_TIE8(f) \
  "+v"(f[0]), "+v"(f[1]), "+v"(f[2]), "+v"(f[3]), "+v"(f[4]), "+v"(f[5]), "+v"(f[6]), "+v"(f[7])

struct Tile {
  int expert, row0, rows, col0;
};

// Tiles are ordered expert-major, then n-tile, then m-tile (m fastest), and the list is cut into 8
// contiguous runs, one per XCD (consecutive block ids go round-robin over the XCDs), so that the
// CUs sharing an L2 work on the same weight panels at the same time.
__device__ __forceinline__ bool find_tile(const int32_t* __restrict__ offsets, int n_exp, int Nout,
                                          int bid, Tile& t) {
  const int n_tiles = (Nout + BN - 1) / BN;
  int m_total = 0;
  for (int i = 0; i < n_exp; ++i) m_total += (offsets[i + 1] - offsets[i] + BM - 1) / BM;
  const int total = m_total * n_tiles;
  const int per = (total + 7) >> 3;
  int tile = (bid & 7) * per + (bid >> 3);
  if ((bid >> 3) >= per || tile >= total) return false;
  int lo = offsets[0];
  for (int i = 0; i < n_exp; ++i) {
    const int hi = offsets[i + 1];
    const int m_tiles = (hi - lo + BM - 1) / BM;
    const int here = m_tiles * n_tiles;
    if (tile < here) {
      const int nt = tile / m_tiles, mt = tile - nt * m_tiles;
      t.expert = i;
      t.row0 = lo + mt * BM;
      t.rows = min(BM, hi - t.row0);
      t.col0 = nt * BN;
      return true;
    }
    tile -= here;
    lo = hi;
  }
  return false;
}

template <bool GELU>
__global__ __launch_bounds__(kThreads) void grouped_gemm_bf16_fast_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, bf16_t* __restrict__ C,
    const int32_t* __restrict__ offsets, int n_exp, int Nout, int K) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];

  Tile tc;
  if (!find_tile(offsets, n_exp, Nout, blockIdx.x, tc)) return;
  const int cols = min(BN, Nout - tc.col0);

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
      (const __attribute__((address_space(3))) unsigned char*)lds));

  // ---- global -> register -> LDS staging ---------------------------------------------------------
  // A tile is 512 rows (256 token, 256 weight) of 128 bytes; one load instruction covers 8 rows, so a
  // tile is 64 instructions, 16 per wavefront.  Wavefronts 0,1 fetch token rows, 2,3 weight rows;
  // instruction n of a wavefront covers rows (wave & 1) * 128 + n * 8 .. + 8 of its operand.
  const bool is_b = wave >= 2;
  const unsigned char* gbase = reinterpret_cast<const unsigned char*>(
      is_b ? B + (static_cast<size_t>(tc.expert) * Nout + tc.col0) * K
           : A + static_cast<size_t>(tc.row0) * K);
  const int row_lim = (is_b ? cols : tc.rows) - 1;
  const int lrow = lane >> 3, piece = lane & 7;
  uint32_t goff[16];   // byte offset of this lane's piece in row n*8 + lrow (rows past the end re-read the last)
#pragma unroll
  for (int n = 0; n < 16; ++n) {
    const int row = (wave & 1) * 128 + n * 8 + lrow;
    goff[n] = (static_cast<uint32_t>(min(row, row_lim)) * K + piece * 8) * 2;
  }
  // LDS write address: row*128 + swizzled piece; rows n*8 + lrow: (row >> 1) & 7 = (n & 1) * 4 + (lrow >> 1)
  uint32_t wr_addr[2];
#pragma unroll
  for (int par = 0; par < 2; ++par) {
    const int sw = (par * 4 + (lrow >> 1)) & 7;
    wr_addr[par] = lds0 + (is_b ? kOperandBytes : 0) + ((wave & 1) * 128 + lrow) * 128 + ((piece ^ sw) << 4);
  }
  u32x4 stage[16];
  auto gload = [&](int n, int t) {   // t: tile index along K
    stage[n] = *reinterpret_cast<const u32x4*>(gbase + goff[n] + static_cast<size_t>(t) * (BK * 2));
  };

  // ---- MFMA operand addresses --------------------------------------------------------------------
  // Lane holds row (lane & 31) of a 32-row fragment and the 8 k-values of piece 2*ks + (lane >> 5).
  const int frow = lane & 31, half = lane >> 5;
  uint32_t tok_addr[4], wgt_addr[4];
#pragma unroll
  for (int ks = 0; ks < 4; ++ks) {
    const int slot = ((2 * ks + half) ^ ((frow >> 1) & 7)) << 4;
    tok_addr[ks] = lds0 + (wm * 128 + frow) * 128 + slot;
    wgt_addr[ks] = lds0 + kOperandBytes + (wn * 128 + frow) * 128 + slot;
  }

  f32x16 acc[4][4];
#pragma unroll
  for (int mi = 0; mi < 4; ++mi)
#pragma unroll
    for (int ni = 0; ni < 4; ++ni)
#pragma unroll
      for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

  bf16x8 f0[8], f1[8];

// The sched_barrier pins the hand-written interleaving of MFMAs and memory operations: without it
// the compiler sinks the fragment reads below the MFMAs (to reuse their registers) and the next
// k-step then waits for LDS.
#define PPMOE_MFMA(f, mi, ni)                                                                        \
  do {                                                                                               \
    __builtin_amdgcn_sched_barrier(0);                                                               \
    acc[mi][ni] = __builtin_amdgcn_mfma_f32_32x32x16_bf16(f[4 + ni], f[mi], acc[mi][ni], 0, 0, 0); \
    __builtin_amdgcn_sched_barrier(0);                                                               \
  } while (0)
#define PPMOE_READ_TOK(f, i, ks, buf) lds_read16<i * 4096>(f[i], tok_addr[ks] + (buf))
#define PPMOE_READ_WGT(f, i, ks, buf) lds_read16<i * 4096>(f[4 + i], wgt_addr[ks] + (buf))
#define PPMOE_WRITE(n, buf) lds_write16<(n) * 1024>(wr_addr[(n) & 1] + (buf), stage[n])
#define PPMOE_WRITE4(q, buf)     \
  do {                           \
    PPMOE_WRITE(4 * q + 0, buf); \
    PPMOE_WRITE(4 * q + 1, buf); \
    PPMOE_WRITE(4 * q + 2, buf); \
    PPMOE_WRITE(4 * q + 3, buf); \
  } while (0)

  // One k-step: 16 MFMAs on `cur`, the 8 fragment reads of the next k-step into `nxt`, and one
  // quarter (4 instructions) of the staging traffic: write quarter Q to LDS, then reload it.
  // RB/WB: byte offsets of the buffer read from / written to.  NKS: k-step the reads are for.
#define PPMOE_STEP(cur, nxt, NKS, RB, Q, WB, LT, DO_READ, DO_STAGE)                                  \
  do {                                                                                               \
    PPMOE_MFMA(cur, 0, 0);                                                                           \
    if (DO_READ) PPMOE_READ_TOK(nxt, 0, NKS, RB);                                                    \
    PPMOE_MFMA(cur, 0, 1);                                                                           \
    if (DO_READ) PPMOE_READ_WGT(nxt, 0, NKS, RB);                                                    \
    PPMOE_MFMA(cur, 1, 0);                                                                           \
    if (DO_READ) PPMOE_READ_TOK(nxt, 1, NKS, RB);                                                    \
    PPMOE_MFMA(cur, 1, 1);                                                                           \
    if (DO_READ) PPMOE_READ_WGT(nxt, 1, NKS, RB);                                                    \
    PPMOE_MFMA(cur, 0, 2);                                                                           \
    if (DO_READ) PPMOE_READ_TOK(nxt, 2, NKS, RB);                                                    \
    PPMOE_MFMA(cur, 0, 3);                                                                           \
    if (DO_READ) PPMOE_READ_WGT(nxt, 2, NKS, RB);                                                    \
    PPMOE_MFMA(cur, 1, 2);                                                                           \
    if (DO_READ) PPMOE_READ_TOK(nxt, 3, NKS, RB);                                                    \
    PPMOE_MFMA(cur, 1, 3);                                                                           \
    if (DO_READ) PPMOE_READ_WGT(nxt, 3, NKS, RB);                                                    \
    PPMOE_MFMA(cur, 2, 0);                                                                           \
    if (DO_STAGE) PPMOE_WRITE(4 * Q + 0, WB);                                                        \
    PPMOE_MFMA(cur, 2, 1);                                                                           \
    if (DO_STAGE) PPMOE_WRITE(4 * Q + 1, WB);                                                        \
    PPMOE_MFMA(cur, 3, 0);                                                                           \
    if (DO_STAGE) PPMOE_WRITE(4 * Q + 2, WB);                                                        \
    PPMOE_MFMA(cur, 3, 1);                                                                           \
    if (DO_STAGE) PPMOE_WRITE(4 * Q + 3, WB);                                                        \
    PPMOE_MFMA(cur, 2, 2);                                                                           \
    if (DO_STAGE) gload(4 * Q + 0, LT);                                                              \
    PPMOE_MFMA(cur, 2, 3);                                                                           \
    if (DO_STAGE) gload(4 * Q + 1, LT);                                                              \
    PPMOE_MFMA(cur, 3, 2);                                                                           \
    if (DO_STAGE) gload(4 * Q + 2, LT);                                                              \
    PPMOE_MFMA(cur, 3, 3);                                                                           \
    if (DO_STAGE) gload(4 * Q + 3, LT);                                                              \
  } while (0)

  const int KT = K / BK;
  const int last = KT - 1;

  // ---- prologue ----------------------------------------------------------------------------------
  // Tile 0 goes through the registers into buffer 0; then tile 1 is loaded, its first quarter written
  // to buffer 1 and replaced by the first quarter of tile 2: the state every loop iteration starts in.
  // Tiles past the end of K are loaded from the last tile instead (never used), which keeps the loop
  // free of branches.
#pragma unroll
  for (int n = 0; n < 16; ++n) gload(n, 0);
  PPMOE_WRITE4(0, 0); PPMOE_WRITE4(1, 0); PPMOE_WRITE4(2, 0); PPMOE_WRITE4(3, 0);
#pragma unroll
  for (int n = 0; n < 16; ++n) gload(n, min(1, last));
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  __builtin_amdgcn_s_barrier();
  PPMOE_READ_TOK(f0, 0, 0, 0); PPMOE_READ_WGT(f0, 0, 0, 0);
  PPMOE_READ_TOK(f0, 1, 0, 0); PPMOE_READ_WGT(f0, 1, 0, 0);
  PPMOE_READ_TOK(f0, 2, 0, 0); PPMOE_READ_WGT(f0, 2, 0, 0);
  PPMOE_READ_TOK(f0, 3, 0, 0); PPMOE_READ_WGT(f0, 3, 0, 0);
  // (after the reads, so that the loop's first wait sees the same 8 reads + 4 writes as every other)
  PPMOE_WRITE4(0, kBufBytes);
#pragma unroll
  for (int n = 0; n < 4; ++n) gload(n, min(2, last));

  // ---- main loop -----------------------------------------------------------------------------------
  // At the top of tile t: buffer t&1 holds tile t (visible to all), f0 <- its k-step 0 (in flight),
  // stage[4..15] hold quarters 1..3 of tile t+1 and stage[0..3] quarter 0 of tile t+2 (in flight),
  // quarter 0 of tile t+1 is already in buffer (t+1)&1.
  for (int t = 0; t < KT; ++t) {
    const uint32_t rb = (t & 1) * kBufBytes, wb = kBufBytes - rb;
    const int lt = min(t + 2, last);
    // LDS operations complete in order: the 8 reads being waited for were always followed by exactly
    // 4 writes, so "at most 4 outstanding" means the reads have landed.
    asm volatile("s_waitcnt lgkmcnt(4)" : PPMOE_TIE8(f0)::"memory");
    PPMOE_STEP(f0, f1, 1, rb, 1, wb, lt, true, true);
    asm volatile("s_waitcnt lgkmcnt(4)" : PPMOE_TIE8(f1)::"memory");
    PPMOE_STEP(f1, f0, 2, rb, 2, wb, lt, true, true);
    asm volatile("s_waitcnt lgkmcnt(4)" : PPMOE_TIE8(f0)::"memory");
    PPMOE_STEP(f0, f1, 3, rb, 3, wb, lt, true, true);
    // Every read of tile t and every write of tile t+1 by this wavefront has completed once
    // lgkmcnt is 0; after the barrier that holds for the whole block.
    asm volatile("s_waitcnt lgkmcnt(0)" : PPMOE_TIE8(f1)::"memory");
    __builtin_amdgcn_s_barrier();
    // k-step 3: prefetch k-step 0 of tile t+1; quarter 0 of tile t+2 goes into the buffer tile t is
    // leaving, and is replaced in the registers by quarter 0 of tile t+3.
    const int lt3 = min(t + 3, last);
    PPMOE_STEP(f1, f0, 0, wb, 0, rb, lt3, true, true);
  }
#undef PPMOE_STEP
#undef PPMOE_WRITE4
#undef PPMOE_WRITE
#undef PPMOE_READ_TOK
#undef PPMOE_READ_WGT
#undef PPMOE_MFMA
  asm volatile("s_waitcnt lgkmcnt(0)" : PPMOE_TIE8(f0)::"memory");

  // ---- epilogue ----------------------------------------------------------------------------------
  // D = W_frag (32 n) x Tok_frag^T (32 m): lane holds token m = lane & 31 and, in register v, output
  // column n = (v / 4) * 8 + (lane >> 5) * 4 + v % 4: four consecutive columns per group of 4.
  // The 128 x 128 sub-tile of a wavefront goes through its own 32 KiB of LDS (rows of 256 bytes,
  // 16-byte chunk c of row r at chunk c ^ (r & 15)) so that global stores are 16 bytes per lane and
  // 256 contiguous bytes per row instead of 8-byte pieces scattered over 32 rows.
  __builtin_amdgcn_s_barrier();   // every wavefront is done with the tile buffers
  const uint32_t epi = lds0 + wave * (128 * 256);
#pragma unroll
  for (int mi = 0; mi < 4; ++mi) {
    const int r = mi * 32 + frow;
#pragma unroll
    for (int ni = 0; ni < 4; ++ni) {
#pragma unroll
      for (int q = 0; q < 4; ++q) {
        float v0 = acc[mi][ni][q * 4 + 0], v1 = acc[mi][ni][q * 4 + 1];
        float v2 = acc[mi][ni][q * 4 + 2], v3 = acc[mi][ni][q * 4 + 3];
        if (GELU) {
          v0 = gelu_tanh(v0);
          v1 = gelu_tanh(v1);
          v2 = gelu_tanh(v2);
          v3 = gelu_tanh(v3);
        }
        const int chunk = ni * 4 + q;   // 16-byte chunk of the 256-byte row; `half` picks its 8-byte half
        const uint32_t a = epi + r * 256 + ((chunk ^ (r & 15)) << 4) + half * 8;
        const uint32_t lo = pack_bf16x2(v0, v1), hi = pack_bf16x2(v2, v3);
        asm volatile("ds_write_b64 %0, %1" : : "v"(a), "v"(static_cast<uint64_t>(lo) | (static_cast<uint64_t>(hi) << 32)) : "memory");
      }
    }
    __builtin_amdgcn_sched_barrier(0);   // one row block at a time keeps the register footprint small
  }
  asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
  // Read back 16 bytes per lane: an instruction covers 4 rows x 256 bytes.
  const int er = lane >> 4, ec = lane & 15;
  const int ncol = cols - wn * 128;   // valid columns of this wavefront's half (may be <= 0)
#pragma unroll 4
  for (int i = 0; i < 32; ++i) {
    const int r = i * 4 + er;
    u32x4 v;
    const uint32_t a = epi + r * 256 + ((ec ^ (r & 15)) << 4);
    asm volatile("ds_read_b128 %0, %1\n\ts_waitcnt lgkmcnt(0)" : "=v"(v) : "v"(a) : "memory");
    const int m = wm * 128 + r;
    if (m < tc.rows && ec * 8 < ncol)
      *reinterpret_cast<u32x4*>(C + static_cast<size_t>(tc.row0 + m) * Nout + tc.col0 + wn * 128 + ec * 8) = v;
  }
}

}  // namespace fast

hipError_t launch_grouped_gemm_fast(bool gelu, const bf16_t* A, const bf16_t* B, bf16_t* C,
                                    const int32_t* offsets, int n_exp, int64_t max_rows, int Nout,
                                    int K, hipStream_t s) {
  using namespace fast;
  static hipError_t attr = [] {
    hipError_t e = hipFuncSetAttribute(
        reinterpret_cast<const void*>(grouped_gemm_bf16_fast_kernel<true>),
        hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
    return hipFuncSetAttribute(reinterpret_cast<const void*>(grouped_gemm_bf16_fast_kernel<false>),
                               hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
  }();
  if (attr != hipSuccess) return attr;
  const int64_t m_tiles = (max_rows + BM - 1) / BM + n_exp;   // upper bound on the sum of ceilings
  const int64_t n_tiles = (Nout + BN - 1) / BN;
  const unsigned grid = static_cast<unsigned>(((m_tiles * n_tiles + 7) / 8) * 8);
  if (gelu)
    grouped_gemm_bf16_fast_kernel<true><<<grid, kThreads, kLdsBytes, s>>>(A, B, C, offsets, n_exp, Nout, K);
  else
    grouped_gemm_bf16_fast_kernel<false><<<grid, kThreads, kLdsBytes, s>>>(A, B, C, offsets, n_exp, Nout, K);
  return hipGetLastError();
}

}  // namespace ppmoe
