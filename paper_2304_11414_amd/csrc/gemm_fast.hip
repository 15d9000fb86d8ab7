// Fast path of the grouped expert GEMMs (Section 3.3.2; FFN = GeLU(X A) B, Section 3.1.3) for bf16
// with K a multiple of 64:
//
//   C[r, n] = act( sum_k A[r, k] * B[i][n, k] ),  offsets[i] <= r < offsets[i+1]
//
// Block tile 256 x 256 x 64, four wavefronts (one per SIMD), each owning a 128 x 128 sub-tile as
// 4 x 4 MFMA 32x32x16 bf16 accumulators (256 accumulator registers).
//
// A 256x256 tile needs 32 bytes per CU per clock from the L2 at full MFMA rate, about what the
// fetch path of a CU sustains, so the loop is built around keeping that path evenly busy:
//   * staging loads are buffer loads of 16 bytes per lane, 8 lanes per row: every request is a whole
//     128-byte line;
//   * exactly one memory instruction (LDS read, LDS write or load) is issued after each MFMA, all
//     through the K loop, never in a burst;
//   * a load stays in flight in registers for two tile times (two sets of staging registers) before
//     it is written to LDS, and LDS holds two tiles (written one tile ahead of use);
//   * one barrier per tile, placed after the third of the four k-steps, when every wavefront has
//     already fetched the last fragments of the current tile: the fragments of the next tile are
//     prefetched behind it, so no LDS latency is exposed at the tile boundary.
//
// LDS layout of a tile buffer: 256 token rows then 256 weight rows of 128 bytes (eight 16-byte
// pieces); piece p of row r sits at slot p ^ ((r >> 1) & 7).  A ds_read_b128 serves 16 lanes per
// cycle (16 consecutive rows, same logical piece) from 64 banks, and with this swizzle they touch 16
// different 16-byte slots; so do the 16 lanes (2 rows x 8 pieces) of a ds_write_b128.
//
// Scheduling: the kernel is persistent (one block per CU; consecutive block ids go round-robin over
// the 8 XCDs, checked once per process with the XCC_ID register).  Row tiles are "big" (up to 256
// rows) or, for the last at most 128 rows of an expert, "small" (computed as 32/64/128 rows x 256
// columns with the four wavefronts side by side: a tail of a few rows costs a few MFMAs, not a tile).
// Big tiles are taken whole, in rounds of the whole chip; the tile list is ordered in blocks of a
// few row tiles x a few column tiles and an XCD runs one block per round, so the CUs sharing an L2
// work on the same panels and neighbouring XCDs on neighbouring blocks.  What is left (big tiles
// when there are fewer than CUs, and the small tiles) is one stream of k-tiles per XCD cut into
// shares (stream-K); an XCD runs its stream between two of its rounds, each XCD at another point of
// the launch, so that this HBM-bound work runs beside the other XCDs' MFMA-bound rounds instead of as
// a phase of the whole chip.  A tile cut between CUs is finished by the CU that holds its first k-tile; the
// others store their partial accumulators to a scratch slot and raise a flag.  Writer and reader of
// a slot sit on the same XCD, so the hand-over goes through their shared L2 without device-scope
// cache maintenance (the device-scope fences are kept as a fallback for any other placement).
//
// A hand-over that does not arrive within the spin limit (the persistent blocks were not all resident:
// another kernel held compute units), or that would come from another XCD's L2, is not waited for:
// the reading CU computes the missing k range itself, so the output tile is always complete and the
// error word only reports lost time.
//
// All LDS traffic is inline assembly with hand-counted lgkmcnt waits, so that the MFMA stream never
// waits for more than it needs; global loads are buffer loads (the compiler counts vmcnt for them).

#include <atomic>
#include <mutex>
#include <type_traits>

#include "common.h"

namespace ppmoe {


namespace fast {

constexpr int BM = 256, BN = 256, BK = 64;
constexpr int kThreads = 256;
constexpr int kOperandBytes = BM * BK * 2;     // 32 KiB
constexpr int kBufBytes = 2 * kOperandBytes;   // 64 KiB: one tile (tokens + weights)
constexpr int kLdsBytes = 2 * kBufBytes;       // 128 KiB

// Reads one accumulator element where it lives (an accumulator register), at this point of the
// program: without it the compiler copies all 256 accumulators to vector registers right after the
// K loop and spills half of them.
__device__ __forceinline__ float read_acc(float a) {
  float v;
  asm volatile("v_accvgpr_read_b32 %0, %1" : "=v"(v) : "a"(a));
  return v;
}

// GeLU, tanh form: 0.5 u (1 + tanh(z)) = u / (1 + exp(-2 z)),  z = sqrt(2/pi) (u + 0.044715 u^3).
// exp2 and the reciprocal are single hardware instructions (about 1 ulp each), ample for a bf16
// result.  Four at a time, stage by stage: the four dependency chains (mul, fma, mul, exp2, add,
// rcp, mul) interleave, so the latency of each instruction is hidden by the other three elements.
__device__ __forceinline__ f32x4 gelu_tanh4(f32x4 u) {
  // (the sched_barriers keep the compiler from folding the stages back into four serial chains)
  f32x4 z, e, r;
#pragma unroll
  for (int i = 0; i < 4; ++i) z[i] = fmaf(0.044715f * u[i], u[i], 1.0f);
#pragma unroll
  for (int i = 0; i < 4; ++i) z[i] = (-2.302208198f * u[i]) * z[i];   // -2 sqrt(2/pi) log2(e) (u + 0.044715 u^3)
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < 4; ++i) e[i] = __builtin_amdgcn_exp2f(z[i]);
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < 4; ++i) e[i] = 1.0f + e[i];
  __builtin_amdgcn_sched_barrier(0);
#pragma unroll
  for (int i = 0; i < 4; ++i) r[i] = __builtin_amdgcn_rcpf(e[i]);
  __builtin_amdgcn_sched_barrier(0);
  return u * r;
}

template <int OFF, typename V>
__device__ __forceinline__ void lds_read16(V& dst, uint32_t addr) {
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

// How a tile is computed.  0: "big", the wavefronts form a 2 x 2 grid of 128 x 128 sub-tiles.
// 1, 2, 4: "small", at most 32, 64, 128 rows: the wavefronts stand side by side, each owning all
// the rows and 64 of the 256 columns (KIND x 2 accumulator blocks instead of 4 x 4), so a tail of a
// few rows costs its share of MFMAs and the fetch of its weight panel, not a whole tile.
__device__ __forceinline__ int tile_kind(int rows, bool small) {
  return !small ? 0 : rows <= 32 ? 1 : rows <= 64 ? 2 : 4;
}

// An expert's rows are cut into m-tiles of BM; its last m-tile is "small" when it has at most
// kSmallRows rows.  The tile list has two parts: all the other ("big") tiles, ordered expert-major,
// in blocks of row tiles x column tiles (see big_tile_at); then the small tiles, ordered
// expert-major, then n-tile.
constexpr int kSmallRows = 128;
constexpr int kMinShare = 16;   // k-tiles: the smallest share of a cut stream a CU is given (8, 12, 24 and 32 measured slower)

__device__ __forceinline__ void expert_tiles(int cnt, int small_rows, int& big_m, int& small) {
  const int m_tiles = (cnt + BM - 1) / BM;
  small = (m_tiles > 0 && cnt - (m_tiles - 1) * BM <= small_rows) ? 1 : 0;
  big_m = m_tiles - small;
}

__device__ __forceinline__ void count_tiles(const int32_t* __restrict__ offsets, int n_exp,
                                            int n_tiles, int small_rows, int& total_big,
                                            int& total_small) {
  total_big = total_small = 0;
  for (int i = 0; i < n_exp; ++i) {
    int big_m, small;
    expert_tiles(offsets[i + 1] - offsets[i], small_rows, big_m, small);
    total_big += big_m * n_tiles;
    total_small += small * n_tiles;
  }
}

// Big tiles of one expert are listed in blocks of hm row tiles x hn column tiles (hm = up to 8,
// hm * hn = the CUs of an XCD), row tile fastest inside a block, blocks along the columns first:
// `cus` consecutive tiles -- what an XCD runs at the same time -- share hm token panels and hn
// weight panels, and the blocks the eight XCDs run at the same time share their token panels.
// (Listing an expert column by column instead gives every CU of an XCD its own token panel: with
// 100 row tiles per expert each token panel was fetched again for every column tile.)
__device__ __forceinline__ Tile big_tile_at(const int32_t* __restrict__ offsets, int n_exp,
                                            int n_tiles, int small_rows, int cus, int tile) {
  Tile t = {0, 0, 1, 0};
  int lo = offsets[0];
  for (int i = 0; i < n_exp; ++i) {
    const int hi = offsets[i + 1];
    int big_m, small;
    expert_tiles(hi - lo, small_rows, big_m, small);
    const int here = big_m * n_tiles;
    if (tile < here) {
      const int hm = min(big_m, 8), hn = max(1, cus / hm);
      const int mb = tile / (hm * n_tiles);              // block row
      const int t2 = tile - mb * hm * n_tiles;
      const int hmb = min(hm, big_m - mb * hm);          // its height (the last one may be lower)
      const int nb = t2 / (hmb * hn);                    // block inside the block row
      const int t3 = t2 - nb * hmb * hn;
      const int n_in = t3 / hmb, m_in = t3 - n_in * hmb;
      const int mt = mb * hm + m_in, nt = nb * hn + n_in;
      t.expert = i;
      t.row0 = lo + mt * BM;
      t.rows = min(BM, hi - t.row0);
      t.col0 = nt * BN;
      return t;
    }
    tile -= here;
    lo = hi;
  }
  return t;
}

__device__ __forceinline__ Tile small_tile_at(const int32_t* __restrict__ offsets, int n_exp,
                                              int n_tiles, int small_rows, int tile) {
  Tile t = {0, 0, 1, 0};
  int lo = offsets[0];
  for (int i = 0; i < n_exp; ++i) {
    const int hi = offsets[i + 1];
    int big_m, small;
    expert_tiles(hi - lo, small_rows, big_m, small);
    if (small) {
      if (tile < n_tiles) {
        t.expert = i;
        t.row0 = lo + big_m * BM;
        t.rows = hi - t.row0;
        t.col0 = tile * BN;
        return t;
      }
      tile -= n_tiles;
    }
    lo = hi;
  }
  return t;
}

// Scratch for tiles cut between CUs: per block one slot of 256 x 256 float accumulators for the
// partial sums it hands over and one flag, plus a second slot where it parks its own partial sums
// when a hand-over it waited for did not arrive (the first slot may still be unread by its reader).
constexpr int kSlotFloats = BM * BN;
constexpr int kSlotsPerBlock = 2;
// Behind the flags and the error word: four 64-bit words in which block 0 leaves the shader-clock
// and wall-clock counters at its start and at its end (what clock the launch ran at).
constexpr int kClockWord = 2 * kMaxPersistentBlocks + 2;   // (32-bit word index in `flags`, 8-byte aligned)
constexpr int kDefaultSpinLimit = 1 << 17;   // polls of a flag (a few tenths of a second) before giving up

// The XCD (accelerator complex die) this wavefront runs on.
__device__ __forceinline__ uint32_t xcc_id() {
  uint32_t v;
  asm volatile("s_getreg_b32 %0, hwreg(HW_REG_XCC_ID, 0, 4)" : "=s"(v));
  return v;
}

// Set-up check of the placement rule the hand-over of partial sums relies on (block b runs on XCD
// b mod 8, so blocks b and b' with b = b' mod 8 share an L2): every block reports where it ran.
__device__ uint32_t g_xcc_of_block[kMaxPersistentBlocks];   // (each device holds its own copy)
__global__ __launch_bounds__(kThreads) void xcc_probe_kernel() {
  if (threadIdx.x == 0) g_xcc_of_block[blockIdx.x] = xcc_id();
}

// FUSE: 0: A and C are the packed tensors.  1: the rows of A are read through a list (packed row r is
// row aux_rows[r] / aux_div of the matrix given as A): the index selection of Algorithm 1 done by
// the loads of the first GEMM.  2: the placement of the expert outputs into the layer output done by
// the stores of the second GEMM: packed row r belongs to assignment a = aux_rows[r] of token
// a / aux_div; if it is that token's only kept pick on this device (aux_inv[token, :] has no other
// entry >= 0; always so with aux_div == 1) it is multiplied by aux_w[a] and stored as row `token` of
// C, which nobody else writes; otherwise it is stored unweighted as packed row r of C2 and left to
// the combine kernel, which has to add it to the token's other picks.
template <bool GELU, int FUSE, int DT>
__global__ __launch_bounds__(kThreads) void grouped_gemm_bf16_fast_kernel(
    const bf16_t* __restrict__ A, const bf16_t* __restrict__ B, bf16_t* __restrict__ C,
    const int32_t* __restrict__ offsets, int n_exp, int Nout, int K, float* __restrict__ slots,
    uint32_t* __restrict__ flags, uint32_t epoch, int same_l2, int spin_limit,
    const int32_t* __restrict__ aux_rows, const float* __restrict__ aux_w, int aux_div,
    const int32_t* __restrict__ aux_inv, bf16_t* __restrict__ C2) {
  extern __shared__ __attribute__((aligned(1024))) unsigned char lds[];
  __shared__ int contrib[kMaxPersistentBlocks / 8 + 1];   // [0] = how many, then the block ids whose slots to add
  __shared__ int contrib_failed;
  const uint32_t my_xcc = xcc_id();
  // A block's flag is down before it can be looked at: whatever the caller's workspace held, a stale
  // word cannot pass for this launch's epoch (the readers poll tens of microseconds from now).
  if (threadIdx.x == 0)
    __hip_atomic_store(flags + blockIdx.x, 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    unsigned long long* cw = reinterpret_cast<unsigned long long*>(flags + kClockWord);
    cw[0] = clock64();
    cw[1] = wall_clock64();
  }

  const int tid = threadIdx.x, lane = tid & 63;
  const int wave = __builtin_amdgcn_readfirstlane(tid >> 6);
  const int wm = wave >> 1, wn = wave & 1;
  const uint32_t lds0 = static_cast<uint32_t>(reinterpret_cast<uintptr_t>(
      (const __attribute__((address_space(3))) unsigned char*)lds));

  // ---- this block's work -----------------------------------------------------------------------
  // Consecutive block ids go round-robin over the 8 XCDs, so `cus` = gridDim/8 blocks share an L2.
  //  * Big tiles are taken whole, in rounds of the whole chip: in round j, XCD x runs the cus tiles
  //    starting at (8 j + x) cus of the tile list, one per CU.  The list is ordered so that those
  //    cus tiles are a block of a few row tiles x a few column tiles (see big_tile_at): they run at
  //    the same time and in step along K, which is what lets the L2 serve a panel once for several
  //    CUs.  What is left after the whole rounds (fewer than 8 cus tiles) is split evenly over the
  //    XCDs: one more, partial round per XCD -- unless an XCD's part is at most a quarter of its
  //    CUs, see below.
  //  * The small tiles (an eighth per XCD), and before them those few left-over big tiles, form one
  //    stream of k-tiles that is cut into shares, so that a 3-row tail of an expert, or one tile more
  //    than the chip has CUs, does not cost a whole tile slot and every CU has work.  A tile cut
  //    this way is finished by the CU that holds its first k-tile.
  const int n_tiles = (Nout + BN - 1) / BN;
  const int KT = K / BK;
  int total_big, total_small;
  const int small_rows = kSmallRows;
  count_tiles(offsets, n_exp, n_tiles, small_rows, total_big, total_small);
  const int xcd = blockIdx.x & 7, cu = blockIdx.x >> 3, cus = gridDim.x >> 3;
  // Big tiles: whole rounds of the chip first -- in round j XCD x takes the cus tiles starting at
  // (8 j + x) cus of the list, so at any time the eight XCDs work on neighbouring blocks -- then the
  // remainder (fewer than 8 cus tiles), an eighth to each XCD.
  const int chip = 8 * cus;
  const int full_rounds = total_big / chip, rem = total_big - full_rounds * chip;
  const int lx0 = full_rounds * chip + static_cast<int>(static_cast<int64_t>(rem) * xcd / 8);
  const int lx1 = full_rounds * chip + static_cast<int>(static_cast<int64_t>(rem) * (xcd + 1) / 8);
  const int sx0 = static_cast<int>(static_cast<int64_t>(total_small) * xcd / 8);
  const int sx1 = static_cast<int>(static_cast<int64_t>(total_small) * (xcd + 1) / 8);
  // The XCD's part of the remainder (r tiles) either runs as one more, partial round, in which
  // cus - r CUs idle for a tile's KT k-tiles, or joins the stream and is cut among all CUs, which
  // costs the hand-over of the big tiles' partial sums (256 KiB each, and an epilogue that waits for
  // them: about 25 k-tiles' time) and, where tiles share panels, the L2's help: the CUs of a stream
  // are not in step along K.  It is cut when it is small (up to a quarter of the CUs: one tile more
  // than the chip has CUs must not cost a round); and, when there is no whole round at all (few tiles
  // per expert: the tiles share little), when the idle time of the partial round would be larger
  // than that price (long contractions).  Measured: with whole rounds before it, cutting 12 tiles of
  // 320 k-tiles per XCD costs 6 % of the launch, running them as a round 3 %.
  const int rem_x = lx1 - lx0;
  const bool cut_big = rem_x > 0 && (rem_x * 4 <= cus ||
                                     (full_rounds == 0 && static_cast<int64_t>(KT) * (cus - rem_x) >= 25 * cus));
  const int rounds = full_rounds + (!cut_big && lx1 > lx0 ? 1 : 0);
  const int stream_big = cut_big ? lx1 - lx0 : 0;                  // big tiles at the head of the stream
  const int64_t units = static_cast<int64_t>(stream_big + sx1 - sx0) * KT;
  // Shares shorter than kMinShare k-tiles are not worth their hand-over: fewer CUs then take part.
  const int takers = static_cast<int>(max(static_cast<int64_t>(1), min(static_cast<int64_t>(cus), units / kMinShare)));
  auto share_begin = [&](int c) -> int64_t { return units * min(c, takers) / takers; };
  // When an XCD runs its share of the stream: before big round `stream_slot` (= rounds: after the
  // last one), the XCDs spread over the launch.  The stream's small tiles are bound by the HBM stream
  // of their weight panels and leave CUs without a share idle; the big tiles are bound by the matrix
  // cores: spread over the XCDs in time, one kind of work runs beside the other instead of as a
  // phase of the whole chip at the end (measured on four workloads: up to 9 % of a launch).
  const int stream_slot = ((7 - xcd) * (rounds + 1)) >> 3;
  int round = 0;
  int64_t u = share_begin(cu);
  const int64_t u_end = share_begin(cu + 1);

  // Staging: a tile is 512 rows (256 token, 256 weight) of 128 bytes; one load instruction covers 8
  // rows, so a tile is 64 instructions, 16 per wavefront.  Wavefronts 0,1 fetch token rows, 2,3
  // weight rows; instruction n of a wavefront covers rows (wave & 1) * 128 + n * 8 .. + 8.
  const bool is_b = wave >= 2;
  const unsigned char* gbase;
  uint32_t goff[16];   // byte offset of this lane's piece in row n*8 + lrow (rows past the end re-read the last)
  f32x16 acc[4][4];

// The sched_barrier pins the hand-written interleaving of MFMAs and memory operations: without it
// the compiler sinks the fragment reads below the MFMAs (to reuse their registers) and the next
// k-step then waits for LDS.
// KIND (a constant of the enclosing segment body) selects the accumulator blocks and fragments in
// use: all 4 x 4 for a big tile, KIND x 2 for a small one.
#define PPMOE_MFMA(f, mi, ni)                                                                        \
  do {                                                                                               \
    __builtin_amdgcn_sched_barrier(0);                                                               \
    if (KIND == 0 || (mi < KIND && ni < 2))                                                          \
      acc[mi][ni] = Elem16<DT>::mfma32(f[4 + ni], f[mi], acc[mi][ni]);                               \
    __builtin_amdgcn_sched_barrier(0);                                                               \
  } while (0)
#define PPMOE_READ_TOK(f, i, ks, buf)                                                  \
  do {                                                                                 \
    if (KIND == 0 || i < KIND) lds_read16<i * 4096>(f[i], tok_a[ks] + (buf));           \
  } while (0)
#define PPMOE_READ_WGT(f, i, ks, buf)                                                  \
  do {                                                                                 \
    if (KIND == 0 || i < 2) lds_read16<i * 4096>(f[4 + i], wgt_a[ks] + (buf));          \
  } while (0)
// S: which of the two sets of staging registers (each holds one tile's share of this wavefront).
#define PPMOE_WRITE(S, n, buf) lds_write16<(n) * 1024>(wr_addr[(n) & 1] + (buf), stage[(S) * 16 + (n)])
#define PPMOE_WRITE4(S, q, buf)     \
  do {                              \
    PPMOE_WRITE(S, 4 * q + 0, buf); \
    PPMOE_WRITE(S, 4 * q + 1, buf); \
    PPMOE_WRITE(S, 4 * q + 2, buf); \
    PPMOE_WRITE(S, 4 * q + 3, buf); \
  } while (0)

  // One k-step: 16 MFMAs on `cur`, the 8 fragment reads of the next k-step into `nxt`, and one
  // quarter (4 instructions) of the staging traffic: write quarter Q of register set S to LDS, then
  // reload it.
  // RB/WB: byte offsets of the buffer read from / written to.  NKS: k-step the reads are for.
  // One memory instruction per MFMA, and never two LDS writes in consecutive slots: four wavefronts
  // writing 1 KiB each in the same 32 cycles exceed what the LDS takes in, and the wavefront then
  // stalls at the next write (measured: 4 writes in 4 consecutive slots cost 56 cycles per k-step,
  // the same 4 writes one every 4 slots cost nothing).  The last LDS instruction of a k-step is a
  // write and every read precedes it: "at most 1 outstanding" means the reads have landed.
#define PPMOE_STEP(cur, nxt, NKS, RB, S, Q, WB, LT, DO_READ, DO_STAGE)                                  \
  do {                                                                                               \
    PPMOE_MFMA(cur, 0, 0);                                                                           \
    if (DO_READ) PPMOE_READ_TOK(nxt, 0, NKS, RB);                                                    \
    PPMOE_MFMA(cur, 0, 1);                                                                           \
    if (DO_READ) PPMOE_READ_WGT(nxt, 0, NKS, RB);                                                    \
    PPMOE_MFMA(cur, 1, 0);                                                                           \
    if (DO_STAGE) PPMOE_WRITE(S, 4 * Q + 0, WB);                                                     \
    PPMOE_MFMA(cur, 1, 1);                                                                           \
    if (DO_READ) PPMOE_READ_TOK(nxt, 1, NKS, RB);                                                    \
    PPMOE_MFMA(cur, 0, 2);                                                                           \
    if (DO_STAGE && stage_live(Q)) gload(S, 4 * Q + 0, LT);                                          \
    PPMOE_MFMA(cur, 0, 3);                                                                           \
    if (DO_READ) PPMOE_READ_WGT(nxt, 1, NKS, RB);                                                    \
    PPMOE_MFMA(cur, 1, 2);                                                                           \
    if (DO_STAGE) PPMOE_WRITE(S, 4 * Q + 1, WB);                                                     \
    PPMOE_MFMA(cur, 1, 3);                                                                           \
    if (DO_READ) PPMOE_READ_TOK(nxt, 2, NKS, RB);                                                    \
    PPMOE_MFMA(cur, 2, 0);                                                                           \
    if (DO_STAGE && stage_live(Q)) gload(S, 4 * Q + 1, LT);                                          \
    PPMOE_MFMA(cur, 2, 1);                                                                           \
    if (DO_READ) PPMOE_READ_WGT(nxt, 2, NKS, RB);                                                    \
    PPMOE_MFMA(cur, 3, 0);                                                                           \
    if (DO_STAGE) PPMOE_WRITE(S, 4 * Q + 2, WB);                                                     \
    PPMOE_MFMA(cur, 3, 1);                                                                           \
    if (DO_READ) PPMOE_READ_TOK(nxt, 3, NKS, RB);                                                    \
    PPMOE_MFMA(cur, 2, 2);                                                                           \
    if (DO_STAGE && stage_live(Q)) gload(S, 4 * Q + 2, LT);                                          \
    PPMOE_MFMA(cur, 2, 3);                                                                           \
    if (DO_READ) PPMOE_READ_WGT(nxt, 3, NKS, RB);                                                    \
    PPMOE_MFMA(cur, 3, 2);                                                                           \
    if (DO_STAGE) PPMOE_WRITE(S, 4 * Q + 3, WB);                                                     \
    PPMOE_MFMA(cur, 3, 3);                                                                           \
    if (DO_STAGE && stage_live(Q)) gload(S, 4 * Q + 3, LT);                                          \
  } while (0)


  // A hand-over that fails (see below) makes the reader put its own partial sums into its own slot
  // and run the rest of the tile's k range as one more segment: resume_tl / resume_kb say which.
  int resume_tl = -1, resume_kb = 0;
  while (resume_tl >= 0 || round < rounds || u < u_end) {
    // ---- one segment: k-tiles [kb, ke) of one output tile ---------------------------------------
    int tl = 0, kb = 0, ke = KT, kind = 0;
    Tile tc;
    asm volatile("" : "+s"(resume_tl), "+s"(resume_kb));   // (uniform values: keep them in scalar registers)
    const bool resumed = resume_tl >= 0;
    if (resumed) {
      tl = resume_tl;
      kb = resume_kb;
      resume_tl = -1;
      tc = tl < stream_big ? big_tile_at(offsets, n_exp, n_tiles, small_rows, cus, lx0 + tl)
                           : small_tile_at(offsets, n_exp, n_tiles, small_rows, sx0 + tl - stream_big);
      kind = tile_kind(tc.rows, tl >= stream_big);
    } else if (round < rounds && !(u < u_end && round >= stream_slot)) {
      const int b = round < full_rounds ? (round * 8 + xcd) * cus + cu : lx0 + cu;
      const bool none = round >= full_rounds && b >= lx1;   // the last round may be partial
      ++round;
      if (none) continue;   // (the stream, if any, still follows)
      tc = big_tile_at(offsets, n_exp, n_tiles, small_rows, cus, b);
    } else {
      tl = static_cast<int>(u / KT);
      kb = static_cast<int>(u - static_cast<int64_t>(tl) * KT);
      ke = static_cast<int>(min(static_cast<int64_t>(KT), kb + (u_end - u)));
      u += ke - kb;
      tc = tl < stream_big ? big_tile_at(offsets, n_exp, n_tiles, small_rows, cus, lx0 + tl)
                           : small_tile_at(offsets, n_exp, n_tiles, small_rows, sx0 + tl - stream_big);
      kind = tile_kind(tc.rows, tl >= stream_big);
    }
    // Per-lane addresses.  They do not depend on the tile, but they are derived here, per segment,
    // from an opaque copy of the lane id: computed once before the segment loop they would all stay
    // live across it (some forty registers, which then spill).
    int lane_s = lane;
    asm volatile("" : "+v"(lane_s));
    const int lrow = lane_s >> 3, piece = lane_s & 7;
    // LDS write address: row*128 + swizzled piece; rows n*8 + lrow: (row >> 1) & 7 = (n & 1) * 4 + (lrow >> 1)
    uint32_t wr_addr[2];
#pragma unroll
    for (int par = 0; par < 2; ++par) {
      const int sw = (par * 4 + (lrow >> 1)) & 7;
      wr_addr[par] = lds0 + (is_b ? kOperandBytes : 0) + ((wave & 1) * 128 + lrow) * 128 + ((piece ^ sw) << 4);
    }
    // MFMA operands: lane holds row (lane_s & 31) of a 32-row fragment and the 8 k-values of piece
    // 2*ks + (lane_s >> 5).
    const int frow = lane_s & 31, half = lane_s >> 5;
    uint32_t tok_addr[4], wgt_addr[4];
#pragma unroll
    for (int ks = 0; ks < 4; ++ks) {
      const int slot = ((2 * ks + half) ^ ((frow >> 1) & 7)) << 4;
      tok_addr[ks] = lds0 + (wm * 128 + frow) * 128 + slot;
      wgt_addr[ks] = lds0 + kOperandBytes + (wn * 128 + frow) * 128 + slot;
    }
    const uint32_t epi = lds0 + wave * (128 * 256);   // this wavefront's 32 KiB for the output transpose

    const int last = ke - 1;
    const int cols = min(BN, Nout - tc.col0);
    const bool gathered = FUSE == 1 && !is_b;
    gbase = reinterpret_cast<const unsigned char*>(
        is_b ? B + (static_cast<size_t>(tc.expert) * Nout + tc.col0) * K
             : A + (gathered ? 0 : static_cast<size_t>(tc.row0) * K));
    const int row_lim = (is_b ? cols : tc.rows) - 1;
    if (gathered) {
#pragma unroll
      for (int n = 0; n < 16; ++n) {
        const int row = (wave & 1) * 128 + n * 8 + lrow;
        const int a = aux_rows[tc.row0 + min(row, row_lim)];
        goff[n] = (static_cast<uint32_t>(aux_div == 1 ? a : a / aux_div) * K + piece * 8) * 2;
      }
    } else {
#pragma unroll
      for (int n = 0; n < 16; ++n) {
        const int row = (wave & 1) * 128 + n * 8 + lrow;
        goff[n] = (static_cast<uint32_t>(min(row, row_lim)) * K + piece * 8) * 2;
      }
    }
#pragma unroll
    for (int mi = 0; mi < 4; ++mi)
#pragma unroll
      for (int ni = 0; ni < 4; ++ni)
#pragma unroll
        for (int v = 0; v < 16; ++v) acc[mi][ni][v] = 0.f;

    // The K loop of one segment, compiled once per tile kind.
    auto run_segment = [&](auto kind_c) __attribute__((always_inline)) {
      constexpr int KIND = decltype(kind_c)::value;
      // Staging registers and fragments belong to the segment: declared outside they would carry
      // their last values across the epilogue wherever a kind leaves some of them unwritten.
      u32x4 stage[32];
      // Buffer loads: a scalar descriptor of the tile's panel (base = its first row), this lane's
      // 32-bit byte offset in a register and the k-tile offset as a scalar -- one address register
      // per lane and no 64-bit vector add per load.  (Offsets are 32-bit: a panel of 256 rows must
      // stay below 2 GiB, i.e. K < 4M.)
      // The descriptor ends with the last valid row of the panel: an offset beyond it (there is none,
      // rows are clamped) would read zeros instead of touching memory.  k-tiles past the end of the
      // segment are loaded through an empty descriptor: every lane is out of range and gets zeros, so
      // the MFMAs of a phantom tile add nothing (the loop runs tiles in pairs).
      // (a gathered panel is the whole matrix: the rows the list names are rows of A, nothing to clamp)
      const int64_t panel_bytes = gathered ? 0x7fffffff : static_cast<int64_t>(row_lim + 1) * K * 2;
      const int n_records = static_cast<int>(panel_bytes < 0x7fffffff ? panel_bytes : 0x7fffffff);
      auto gload = [&](int set, int n, int t) {   // t: tile index along K
        const __amdgpu_buffer_rsrc_t rsrc = __builtin_amdgcn_make_buffer_rsrc(
            const_cast<unsigned char*>(gbase), 0, t <= last ? n_records : 0, 0x00020000);
        stage[set * 16 + n] = __builtin_amdgcn_raw_buffer_load_b128(rsrc, goff[n], t * (BK * 2), 0);
      };
      typename Elem16<DT>::vec8 f0[8], f1[8];
      // Small tile: every wavefront reads the token rows from row 0 and its own 64 weight rows.
      // (the shifts are made opaque so that the shifted addresses are computed here, per segment, and
      // not once per kind before the segment loop, where they would be live across everything)
      uint32_t tok_a[4], wgt_a[4];
      uint32_t tok_shift = KIND ? wm * (128 * 128) : 0, wgt_shift = KIND ? (wave * 64 - wn * 128) * 128 : 0;
      asm volatile("" : "+s"(tok_shift), "+s"(wgt_shift));
#pragma unroll
      for (int ks = 0; ks < 4; ++ks) {
        tok_a[ks] = tok_addr[ks] - tok_shift;
        wgt_a[ks] = wgt_addr[ks] + wgt_shift;
      }
      // Token rows are staged 32 at a time by wavefront 0 (quarter q of its loads = rows 32q..32q+31):
      // a small tile only fetches the row blocks it has (wavefront 1 stages rows 128..255: none).
      auto stage_live = [&](int q) -> bool { return KIND == 0 || is_b || (wave == 0 && q < KIND); };

      // ---- prologue ------------------------------------------------------------------------------
      // Two sets of staging registers: a load stays in flight for two tile times before it is written
      // to LDS.  Set i & 1 holds tile kb + i (i = t - kb).  Here: tile kb goes through set 0 into
      // buffer 0; sets 1 and 0 are loaded with tiles kb+1 and kb+2; quarter 0 of tile kb+1 is written
      // to buffer 1 and replaced by quarter 0 of tile kb+3: the state every loop iteration starts in.
      // Tiles past the end of the segment read as zeros, which keeps the loop free of branches.
      auto gload_tile = [&](int set, int t) {
#pragma unroll
        for (int q = 0; q < 4; ++q)
          if (stage_live(q)) {
#pragma unroll
            for (int n = 4 * q; n < 4 * q + 4; ++n) gload(set, n, t);
          }
      };
      gload_tile(0, kb);
      __builtin_amdgcn_s_barrier();   // the previous segment's output transpose is out of LDS
      PPMOE_WRITE4(0, 0, 0); PPMOE_WRITE4(0, 1, 0); PPMOE_WRITE4(0, 2, 0); PPMOE_WRITE4(0, 3, 0);
      gload_tile(1, kb + 1);
      gload_tile(0, kb + 2);
      asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
      __builtin_amdgcn_s_barrier();
      PPMOE_READ_TOK(f0, 0, 0, 0); PPMOE_READ_WGT(f0, 0, 0, 0);
      PPMOE_READ_TOK(f0, 1, 0, 0); PPMOE_READ_WGT(f0, 1, 0, 0);
      PPMOE_READ_TOK(f0, 2, 0, 0); PPMOE_READ_WGT(f0, 2, 0, 0);
      PPMOE_READ_TOK(f0, 3, 0, 0); PPMOE_READ_WGT(f0, 3, 0, 0);
      // (after the reads: the loop's first wait, "at most 1 outstanding", then covers them)
      PPMOE_WRITE4(1, 0, kBufBytes);
      if (stage_live(0)) {
#pragma unroll
        for (int n = 0; n < 4; ++n) gload(1, n, kb + 3);
      }

      // ---- main loop -----------------------------------------------------------------------------
      // At the top of tile t (i = t - kb): buffer i&1 holds tile t (visible to all), f0 <- its k-step
      // 0 (in flight); quarter 0 of tile t+1 is already in buffer (i+1)&1; set (i+1)&1 holds quarters
      // 1..3 of tile t+1 and quarter 0 of tile t+3; set i&1 holds tile t+2 (all in flight or landed).
      // TILE(t, RB, WB, SA, SB): RB/WB the buffers of tiles t / t+1, SA = (i+1)&1, SB = i&1.
#define PPMOE_TILE(t, RB, WB, SA, SB)                                                                \
  do {                                                                                               \
    const int lt = (t) + 3;                                                                          \
    /* LDS operations complete in order: the reads being waited for were always followed by      */ \
    /* exactly one write, so "at most 1 outstanding" means the reads have landed.                 */ \
    asm volatile("s_waitcnt lgkmcnt(1)" : PPMOE_TIE8(f0)::"memory");                                 \
    PPMOE_STEP(f0, f1, 1, RB, SA, 1, WB, lt, true, true);                                            \
    asm volatile("s_waitcnt lgkmcnt(1)" : PPMOE_TIE8(f1)::"memory");                                 \
    PPMOE_STEP(f1, f0, 2, RB, SA, 2, WB, lt, true, true);                                            \
    asm volatile("s_waitcnt lgkmcnt(1)" : PPMOE_TIE8(f0)::"memory");                                 \
    PPMOE_STEP(f0, f1, 3, RB, SA, 3, WB, lt, true, true);                                            \
    /* Every read of tile t and every write of tile t+1 by this wavefront has completed once     */ \
    /* lgkmcnt is 0; after the barrier that holds for the whole block.                            */ \
    asm volatile("s_waitcnt lgkmcnt(0)" : PPMOE_TIE8(f1)::"memory");                                 \
    __builtin_amdgcn_s_barrier();                                                                    \
    /* k-step 3: prefetch k-step 0 of tile t+1; quarter 0 of tile t+2 goes into the buffer tile t */ \
    /* is leaving, and is replaced in the registers by quarter 0 of tile t+4.                     */ \
    const int lt4 = (t) + 4;                                                                         \
    PPMOE_STEP(f1, f0, 0, WB, SB, 0, RB, lt4, true, true);                                           \
  } while (0)
      for (int t = kb; t < ke; t += 2) {   // (a segment of odd length ends with a phantom tile of zeros)
        PPMOE_TILE(t, 0, kBufBytes, 1, 0);
        PPMOE_TILE(t + 1, kBufBytes, 0, 0, 1);
      }
#undef PPMOE_TILE
      asm volatile("s_waitcnt lgkmcnt(0)" : PPMOE_TIE8(f0)::"memory");
    };
    if (kind == 0) run_segment(std::integral_constant<int, 0>{});
    else if (kind == 1) run_segment(std::integral_constant<int, 1>{});
    else if (kind == 2) run_segment(std::integral_constant<int, 2>{});
    else run_segment(std::integral_constant<int, 4>{});

    // A segment that does not hold the first k-tile of its output tile hands its partial sums to the
    // CU that does (through this block's scratch slot) and raises its flag: mode 1.  The one that
    // holds it writes the output tile (mode 0), after adding the partial sums of the CUs after it, if
    // the rest of the k range went there (their first segment, which they finished long ago).  If
    // those do not arrive it takes nobody's: it parks its own partial sums in its own slot (mode 2,
    // no flag) and runs the rest of the k range as one more segment, which ends by adding them back.
    int mode = (kb > 0 && !resumed) ? 1 : 0;
    int n_contrib = 0;
    if (resumed) {
      if (tid == 0) {
        contrib[0] = 1;
        contrib[1] = kMaxPersistentBlocks + blockIdx.x;   // its parking slot
      }
      __syncthreads();
      n_contrib = 1;   // (this CU's own stores, complete since the barrier that followed them)
    } else if (mode == 0 && ke < KT) {
      if (tid == 0) {
        // One thread lists the CUs after this one whose share begins inside this tile (skipping empty
        // shares) and polls their flags (relaxed loads that go to L2, no cache maintenance in the loop).
        int n = 0, failed = 0;
        for (int c2 = cu + 1; c2 < cus && share_begin(c2) < static_cast<int64_t>(tl + 1) * KT; ++c2) {
          if (share_begin(c2 + 1) == share_begin(c2)) continue;
          const int b2 = (c2 << 3) | xcd;
          contrib[++n] = b2;
          int spins = 0;
          uint32_t f = 0;
          bool up = false;
          while (spins < spin_limit) {
            f = __hip_atomic_load(flags + b2, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
            if ((f >> 4) == epoch) {
              up = true;
              break;
            }
            ++spins;
            __builtin_amdgcn_s_sleep(16);
          }
          if (!up) {   // not delivered in time (the writer's block may not even be resident yet)
            failed = 1;
            flags[kMaxPersistentBlocks] = kGemmErrorMagic | 1u;
            break;
          }
          if (same_l2 && (f & 15u) != my_xcc) {
            // The partial sums sit in another XCD's L2 and their writer released them at workgroup
            // scope only (the set-up check of the placement was wrong): they cannot be read safely.
            failed = 1;
            flags[kMaxPersistentBlocks] = kGemmErrorMagic | 2u;
            break;
          }
        }
        contrib[0] = n;
        contrib_failed = failed;
      }
      __syncthreads();
      if (contrib_failed) {
        mode = 2;
      } else {
        // Once per thread, after the flags are up.  Within an XCD the partial sums are in the shared L2
        // (stores write through the L1, and this CU has never read these lines since its L1 was
        // invalidated at the start of the kernel), so ordering against the barrier is all it takes;
        // the device-scope acquire invalidates the L2, which then misses on every panel being streamed.
        if (same_l2)
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "workgroup");
        else
          __builtin_amdgcn_fence(__ATOMIC_ACQUIRE, "agent");
        n_contrib = contrib[0];
      }
    }

    // Per-segment opaque copies: they stop the compiler from hoisting the address arithmetic of the
    // code below out of the segment loop, where it would cost a few hundred live registers.
    uint32_t epi_l = epi;
    int tid_l = tid;
    asm volatile("" : "+v"(epi_l), "+v"(tid_l));
    // Where this wavefront's accumulator blocks sit in the tile (see tile_kind).
    const int row_base = kind ? 0 : wm * 128, col_base = kind ? wave * 64 : wn * 128;
    const int ni_lim = kind ? 2 : 4, wave_cols = kind ? 64 : 128;

    int my_slot_id = (mode == 2 ? kMaxPersistentBlocks : 0) + static_cast<int>(blockIdx.x);
    asm volatile("" : "+s"(my_slot_id));
    f32x4* my_slot = reinterpret_cast<f32x4*>(slots + static_cast<size_t>(my_slot_id) * kSlotFloats) + tid_l;

    // ---- epilogue --------------------------------------------------------------------------------
    // D = W_frag (32 n) x Tok_frag^T (32 m): lane holds token m = lane & 31 and, in register v,
    // output column n = (v / 4) * 8 + (lane >> 5) * 4 + v % 4: four consecutive columns per group.
    // The 128 x 128 sub-tile of a wavefront goes through its own 32 KiB of LDS (rows of 256 bytes,
    // 16-byte chunk c of row r at chunk c ^ (r & 15)) so that global stores are 16 bytes per lane
    // and 256 contiguous bytes per row instead of 8-byte pieces scattered over 32 rows.
    // The accumulators are read in exactly one place (one 32x32 block at a time), whichever way
    // they go: that keeps them in the accumulator registers until then.
    __builtin_amdgcn_s_barrier();   // every wavefront is done with the tile buffers
    // FUSE == 2: where packed row r goes.  >= 0: row of C (the token; r is its only kept pick here);
    // < 0: ~r, packed row r of C2.
    auto placed_row = [&](int r, int& a_out) -> int {
      const int a = aux_rows[r];
      a_out = a;
      if (aux_div == 1) return a;
      const int t = a / aux_div;
      int kept = 0;
      for (int j = 0; j < aux_div; ++j) kept += aux_inv[t * aux_div + j] >= 0;
      return kept == 1 ? t : ~r;
    };
    float row_w[4] = {1.f, 1.f, 1.f, 1.f};   // FUSE == 2: gate weight of this lane's row of each row block
    if (FUSE == 2 && mode == 0) {
#pragma unroll
      for (int mi = 0; mi < 4; ++mi) {
        const int row = min(row_base + mi * 32 + frow, tc.rows - 1);
        int a;
        const int dst = placed_row(tc.row0 + row, a);
        row_w[mi] = dst >= 0 ? aux_w[a] : 1.f;
      }
    }
#pragma unroll
    for (int mi = 0; mi < 4; ++mi) {
#pragma unroll
      for (int ni = 0; ni < 4; ++ni) {
        f32x4 v[4];
#pragma unroll
        for (int q = 0; q < 4; ++q)
#pragma unroll
          for (int e = 0; e < 4; ++e) v[q][e] = read_acc(acc[mi][ni][q * 4 + e]);
        // Blocks of 32 rows with no valid row are neither sent nor fetched (a 3-row tail tile moves an
        // eighth of a slot).
        const bool live = row_base + mi * 32 < tc.rows && ni < ni_lim;
        if (mode != 0) {
          if (live) {
#pragma unroll
            for (int q = 0; q < 4; ++q) my_slot[((mi * 4 + ni) * 4 + q) * kThreads] = v[q];
          }
        } else {
          // Partial sums are added in CU order (fixed summation order); the loads of 8 CUs' slots
          // go out together, so the wait is one memory latency per 8 CUs, not per CU.
          for (int c0 = 0; live && c0 < n_contrib; c0 += 8) {
            f32x4 p[8][4];
#pragma unroll
            for (int j = 0; j < 8; ++j) {
              const bool has = c0 + j < n_contrib;
              const int b2 = contrib[1 + min(c0 + j, n_contrib - 1)];
              const f32x4* slot = reinterpret_cast<const f32x4*>(slots + static_cast<size_t>(b2) * kSlotFloats) + tid_l;
#pragma unroll
              for (int q = 0; q < 4; ++q)
                p[j][q] = has ? slot[((mi * 4 + ni) * 4 + q) * kThreads] : f32x4{0.f, 0.f, 0.f, 0.f};
            }
#pragma unroll
            for (int j = 0; j < 8; ++j)
#pragma unroll
              for (int q = 0; q < 4; ++q) v[q] += p[j][q];
          }
          const int r = mi * 32 + frow;
#pragma unroll
          for (int q = 0; live && q < 4; ++q) {
            f32x4 w = v[q];
            if (GELU) w = gelu_tanh4(w);
            if (FUSE == 2) w *= row_w[mi];
            const int chunk = ni * 4 + q;   // 16-byte chunk of the 256-byte row; `half` picks its 8-byte half
            const uint32_t a = epi_l + r * 256 + ((chunk ^ (r & 15)) << 4) + half * 8;
            const uint32_t lo = Elem16<DT>::pack2(w[0], w[1]), hi = Elem16<DT>::pack2(w[2], w[3]);
            asm volatile("ds_write_b64 %0, %1" : : "v"(a), "v"(static_cast<uint64_t>(lo) | (static_cast<uint64_t>(hi) << 32)) : "memory");
          }
        }
        __builtin_amdgcn_sched_barrier(0);   // one 32x32 block at a time keeps the register footprint small
      }
    }
    if (mode == 2) {
      // Parked: the stores are in the L2 once vmcnt is 0 (this CU's L1 holds no line of its own
      // slot: it has not read it in this launch); the block meets, then goes on with the same tile.
      asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
      __syncthreads();
      resume_tl = tl;
      resume_kb = ke;
      continue;
    }
    if (mode == 1) {
      // Release: every thread makes its own stores visible device-wide, then the block meets, then
      // one thread raises the flag (a relaxed store is enough after the fences).
      // (Within an XCD: the stores have reached the shared L2 once vmcnt is 0.  The device-scope
      // release would write back every dirty line of the L2 -- the output tiles -- once per hand-over.)
      if (same_l2) {
        asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "workgroup");
      } else {
        __builtin_amdgcn_fence(__ATOMIC_RELEASE, "agent");
      }
      __syncthreads();
      if (tid == 0) {
        uint32_t up = (epoch << 4) | my_xcc;
        asm volatile("" : "+s"(up));   // (formed here: hoisted out of the segment loop it would cost a vector register)
        __hip_atomic_store(flags + blockIdx.x, up, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
      }
      continue;
    }
    asm volatile("s_waitcnt lgkmcnt(0)" ::: "memory");
    if (n_contrib > 0 && !resumed) {
      // every thread has read the partial sums: lower the flags (the scratch may be reused by a
      // replay of the same launch, whose flags carry the same value)
      __syncthreads();
      if (tid == 0)
        for (int i = 1; i <= n_contrib; ++i)
          __hip_atomic_store(flags + contrib[i], 0u, __ATOMIC_RELAXED, __HIP_MEMORY_SCOPE_AGENT);
    }
    // Read back 16 bytes per lane: an instruction covers 4 rows x 256 bytes.
    const int er = (tid_l & 63) >> 4, ec = tid_l & 15;
    const int ncol = min(cols - col_base, wave_cols);   // valid columns of this wavefront's part (may be <= 0)
    const int nrow = tc.rows - row_base;                // valid rows of it (may be <= 0)
    bf16_t* cbase = C + static_cast<size_t>(tc.row0 + row_base) * Nout + tc.col0 + col_base + ec * 8;
    for (int i0 = 0; i0 < 32 && i0 * 4 < nrow; i0 += 8) {   // 8 reads in flight, then their 8 stores
      u32x4 v[8];
#pragma unroll
      for (int j = 0; j < 8; ++j) {
        const int r = (i0 + j) * 4 + er;
        const uint32_t a = epi_l + r * 256 + ((ec ^ (r & 15)) << 4);
        asm volatile("ds_read_b128 %0, %1" : "=v"(v[j]) : "v"(a) : "memory");
      }
      asm volatile("s_waitcnt lgkmcnt(0)"
                   : "+v"(v[0]), "+v"(v[1]), "+v"(v[2]), "+v"(v[3]), "+v"(v[4]), "+v"(v[5]), "+v"(v[6]), "+v"(v[7])
                   :
                   : "memory");
      if (FUSE == 2) {
        int dst[8];
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          int a;
          dst[j] = placed_row(tc.row0 + row_base + min((i0 + j) * 4 + er, max(nrow, 1) - 1), a);
        }
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int r = (i0 + j) * 4 + er;
          if (r < nrow && ec * 8 < ncol) {
            bf16_t* base = dst[j] >= 0 ? C : C2;
            const int row = dst[j] >= 0 ? dst[j] : ~dst[j];
            *reinterpret_cast<u32x4*>(base + static_cast<size_t>(row) * Nout + tc.col0 + col_base + ec * 8) = v[j];
          }
        }
      } else {
#pragma unroll
        for (int j = 0; j < 8; ++j) {
          const int r = (i0 + j) * 4 + er;
          if (r < nrow && ec * 8 < ncol)
            *reinterpret_cast<u32x4*>(cbase + static_cast<size_t>(r) * Nout) = v[j];
        }
      }
    }
  }
  if (blockIdx.x == 0 && threadIdx.x == 0) {
    unsigned long long* cw = reinterpret_cast<unsigned long long*>(flags + kClockWord);
    cw[2] = clock64();
    cw[3] = wall_clock64();
  }
#undef PPMOE_STEP
#undef PPMOE_WRITE4
#undef PPMOE_WRITE
#undef PPMOE_READ_TOK
#undef PPMOE_READ_WGT
#undef PPMOE_MFMA
}

}  // namespace fast

hipError_t read_gemm_error_word(const void* workspace, uint32_t* word, hipStream_t s) {
  const float* slots = static_cast<const float*>(workspace);
  const uint32_t* flags = reinterpret_cast<const uint32_t*>(
      slots + static_cast<size_t>(fast::kSlotsPerBlock) * kMaxPersistentBlocks * fast::kSlotFloats);
  hipError_t e = hipMemcpyAsync(word, flags + kMaxPersistentBlocks, sizeof(uint32_t),
                                hipMemcpyDeviceToHost, s);
  if (e != hipSuccess) return e;
  e = hipStreamSynchronize(s);
  if (e != hipSuccess) return e;
  if ((*word & 0xffffff00u) == kGemmErrorMagic) {   // reported once: lower it again
    static const uint32_t zero = 0;
    e = hipMemcpyAsync(const_cast<uint32_t*>(flags) + kMaxPersistentBlocks, &zero, sizeof(uint32_t),
                       hipMemcpyHostToDevice, s);
    if (e != hipSuccess) return e;
    e = hipStreamSynchronize(s);
  }
  return e;
}

// Shader-clock and wall-clock ticks block 0 of the last fast-path launch on this workspace counted
// between its start and its end.  Synchronises the stream.
hipError_t read_gemm_clock_words(const void* workspace, uint64_t* shader_ticks, uint64_t* wall_ticks,
                                 hipStream_t s) {
  const float* slots = static_cast<const float*>(workspace);
  const uint32_t* flags = reinterpret_cast<const uint32_t*>(
      slots + static_cast<size_t>(fast::kSlotsPerBlock) * kMaxPersistentBlocks * fast::kSlotFloats);
  uint64_t w[4] = {0, 0, 0, 0};
  hipError_t e = hipMemcpyAsync(w, flags + fast::kClockWord, sizeof(w), hipMemcpyDeviceToHost, s);
  if (e != hipSuccess) return e;
  e = hipStreamSynchronize(s);
  if (e != hipSuccess) return e;
  *shader_ticks = w[2] - w[0];
  *wall_ticks = w[3] - w[1];
  return hipSuccess;
}

size_t grouped_gemm_fast_workspace_bytes() {
  // slots, flags (+1 word: the error word), and inside the padding the four clock words
  return static_cast<size_t>(fast::kSlotsPerBlock) * kMaxPersistentBlocks * fast::kSlotFloats * sizeof(float) +
         (2 * kMaxPersistentBlocks + 1) * sizeof(uint32_t) + 256;
}

// ---- per-device set-up --------------------------------------------------------------------------
// Once per device: the dynamic-LDS attribute of the kernels, the number of persistent blocks, and the
// placement check (do blocks b and b + 8 share an XCD, as the workgroup-scope hand-over assumes?).
// The check launches a probe and waits for it, so it is the one thing here that synchronises; it
// runs from moe_init, or from the first launch on a device that finds it not done -- unless that
// launch is being captured into a graph, in which case the launch uses device-scope fences and
// leaves the check for later.
namespace {

constexpr int kMaxDevices = 64;
struct FastSetup {
  bool attrs = false;   // kernel attributes set, `blocks` valid
  bool probed = false;  // same_l2 valid
  int blocks = 0;
  int same_l2 = 0;
};
FastSetup g_setup[kMaxDevices];
std::mutex g_setup_mutex;
std::atomic<int> g_force_device_scope{0};
std::atomic<int> g_spin_limit{fast::kDefaultSpinLimit};

hipError_t setup_attrs(FastSetup& st, int dev) {
  using namespace fast;
  if (st.attrs) return hipSuccess;
  const void* kernels[] = {
      reinterpret_cast<const void*>(grouped_gemm_bf16_fast_kernel<true, 0, MOE_BF16>),
      reinterpret_cast<const void*>(grouped_gemm_bf16_fast_kernel<false, 0, MOE_BF16>),
      reinterpret_cast<const void*>(grouped_gemm_bf16_fast_kernel<true, 1, MOE_BF16>),
      reinterpret_cast<const void*>(grouped_gemm_bf16_fast_kernel<false, 2, MOE_BF16>),
      reinterpret_cast<const void*>(grouped_gemm_bf16_fast_kernel<true, 0, MOE_F16>),
      reinterpret_cast<const void*>(grouped_gemm_bf16_fast_kernel<false, 0, MOE_F16>),
      reinterpret_cast<const void*>(grouped_gemm_bf16_fast_kernel<true, 1, MOE_F16>),
      reinterpret_cast<const void*>(grouped_gemm_bf16_fast_kernel<false, 2, MOE_F16>)};
  for (const void* k : kernels) {
    hipError_t e = hipFuncSetAttribute(k, hipFuncAttributeMaxDynamicSharedMemorySize, kLdsBytes);
    if (e != hipSuccess) return e;
  }
  int cus = 0;
  hipError_t e = hipDeviceGetAttribute(&cus, hipDeviceAttributeMultiprocessorCount, dev);
  if (e != hipSuccess) return e;
  if (cus > kMaxPersistentBlocks) cus = kMaxPersistentBlocks;
  st.blocks = cus & ~7;   // one block per CU, the same number on each of the 8 XCDs
  if (st.blocks < 8) return hipErrorInvalidConfiguration;
  st.attrs = true;
  return hipSuccess;
}

// Launches the placement probe on `s` and waits for it.  Must not be called while `s` is capturing.
hipError_t setup_probe(FastSetup& st, hipStream_t s) {
  if (st.probed) return hipSuccess;
  uint32_t host[kMaxPersistentBlocks];
  fast::xcc_probe_kernel<<<st.blocks, fast::kThreads, 0, s>>>();
  hipError_t e = hipGetLastError();
  if (e != hipSuccess) return e;
  e = hipMemcpyFromSymbolAsync(host, HIP_SYMBOL(fast::g_xcc_of_block), st.blocks * sizeof(uint32_t), 0,
                               hipMemcpyDeviceToHost, s);
  if (e != hipSuccess) return e;
  e = hipStreamSynchronize(s);
  if (e != hipSuccess) return e;
  st.same_l2 = 1;
  for (int b = 8; b < st.blocks; ++b)
    if (host[b] != host[b & 7]) st.same_l2 = 0;
  st.probed = true;
  return hipSuccess;
}

}  // namespace

hipError_t grouped_gemm_fast_init(hipStream_t s) {
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  std::lock_guard<std::mutex> lock(g_setup_mutex);
  e = setup_attrs(g_setup[dev], dev);
  if (e != hipSuccess) return e;
  return setup_probe(g_setup[dev], s);
}

void grouped_gemm_fast_set_handover(int force_device_scope, int spin_limit) {
  if (force_device_scope >= 0) g_force_device_scope = force_device_scope ? 1 : 0;
  if (spin_limit >= 0) g_spin_limit = spin_limit;
}

hipError_t launch_grouped_gemm_fast(int in_dtype, bool gelu, const bf16_t* A, const bf16_t* B, bf16_t* C,
                                    const int32_t* offsets, int n_exp, int64_t max_rows, int Nout,
                                    int K, void* workspace, hipStream_t s, int fuse,
                                    const int32_t* aux_rows, const float* aux_w, int aux_div,
                                    const int32_t* aux_inv, bf16_t* C2) {
  using namespace fast;
  int dev = 0;
  hipError_t e = hipGetDevice(&dev);
  if (e != hipSuccess) return e;
  if (dev < 0 || dev >= kMaxDevices) return hipErrorInvalidDevice;
  int blocks = 0, same_l2 = 0;
  {
    std::lock_guard<std::mutex> lock(g_setup_mutex);
    FastSetup& st = g_setup[dev];
    e = setup_attrs(st, dev);
    if (e != hipSuccess) return e;
    if (!st.probed) {
      hipStreamCaptureStatus cap = hipStreamCaptureStatusNone;
      e = hipStreamIsCapturing(s, &cap);
      if (e != hipSuccess) return e;
      if (cap == hipStreamCaptureStatusNone) {
        e = setup_probe(st, s);
        if (e != hipSuccess) return e;
      }
    }
    blocks = st.blocks;
    same_l2 = st.probed ? st.same_l2 : 0;   // unknown placement: device-scope fences are always right
  }
  if (g_force_device_scope.load()) same_l2 = 0;
  const int spin_limit = g_spin_limit.load();
  static std::atomic<uint32_t> launches{0};
  // 28 bits (the flag word also carries the XCD id), spread over the word so that small integers
  // left in a recycled workspace do not look like an epoch; 0 means "flag down".
  uint32_t epoch = (++launches * 0x9E3779B1u) >> 4;
  if (epoch == 0) epoch = (++launches * 0x9E3779B1u) >> 4;
  float* slots = static_cast<float*>(workspace);
  uint32_t* flags = reinterpret_cast<uint32_t*>(
      slots + static_cast<size_t>(kSlotsPerBlock) * kMaxPersistentBlocks * kSlotFloats);
  (void)max_rows;
  // fuse: 0 none; 1 rows of A through aux_rows (first GEMM only); 2 rows of the result placed through
  // aux_rows (second GEMM only; with aux_div > 1 it needs the inverse permutation and a place for
  // the rows it cannot place)
  if ((fuse == 1 && !gelu) || (fuse == 2 && gelu) || fuse < 0 || fuse > 2 ||
      (fuse != 0 && aux_rows == nullptr) || (fuse == 2 && aux_w == nullptr) || aux_div < 1 ||
      (fuse == 2 && aux_div != 1 && (aux_inv == nullptr || C2 == nullptr)))
    return hipErrorInvalidValue;
#define PPMOE_LAUNCH_DT(G, F, DT)                                                     \
  grouped_gemm_bf16_fast_kernel<G, F, DT><<<blocks, kThreads, kLdsBytes, s>>>(        \
      A, B, C, offsets, n_exp, Nout, K, slots, flags, epoch, same_l2, spin_limit, aux_rows, aux_w, aux_div, \
      aux_inv, C2)
#define PPMOE_LAUNCH(G, F)                            \
  do {                                                \
    if (in_dtype == MOE_F16) PPMOE_LAUNCH_DT(G, F, MOE_F16); \
    else PPMOE_LAUNCH_DT(G, F, MOE_BF16);             \
  } while (0)
  if (fuse == 1) PPMOE_LAUNCH(true, 1);
  else if (fuse == 2) PPMOE_LAUNCH(false, 2);
  else if (gelu) PPMOE_LAUNCH(true, 0);
  else PPMOE_LAUNCH(false, 0);
#undef PPMOE_LAUNCH_DT
#undef PPMOE_LAUNCH
  return hipGetLastError();
}

}  // namespace ppmoe
