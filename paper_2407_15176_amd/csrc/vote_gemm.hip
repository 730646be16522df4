// Vote selection for a chunk of query rows: the per-head top-k lists of every (query row,
// query head) (paper, Method, "Full-Context Cache Selection", last paragraph: each head and
// each query votes with its own top-k) against the whole middle of the key cache are one
// dense contraction per KV head, [M * G columns] x [N_mid keys] x [D], so it runs on the
// matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation) with the top-k fused behind it:
// no score is ever written.  bf16 storage makes every head's query an exact MFMA operand, so
// unlike the group-sum contraction there is no hi/lo split and the executed matrix work
// equals the algorithmic 2 * M * Hq * N_mid * D.
//
// Tiling: a workgroup of 8 waves (two per SIMD) owns 512 columns ((query row, head) pairs,
// query-major; 256 for a short chunk or lists of 8) of one KV head and walks key tiles of 128
// rows staged in LDS (four buffers, 272-byte row pitch, filled by loads that go from memory
// straight into LDS).  Keys are the A operand, so a lane of a 32x32 block holds ONE column and 16
// keys: the running top-k list of a column belongs to the lane that owns it (in registers), and
// a block costs a maximum over 16 scores and one comparison unless a score enters the list.
// Wave cw takes the two column blocks 2 cw, 2 cw + 1 (their 2 x 8 query operands stay in
// registers) and all four key blocks of a tile.  Its work is a chain of phases (key block,
// column block): while the matrix pipe works on phase q + 1 the wave filters the scores of
// phase q (two accumulators), both column blocks of a key block share one read of its rows from
// LDS, and the rows of the next key block arrive behind the matrix instructions that read the
// current ones; the first phase of tile t + 1 is in the pipe before the workgroup meets at the
// barrier that ends step t.  The second wave of a SIMD covers what this leaves open: an
// insertion into a list (rare, long, divergent) and the wait at the barrier.  The two partial
// lists of a column (the lane halves) are merged through LDS at the end.  With few query rows
// the keys are also split over blockIdx.z so that the chip is filled; every workgroup writes one
// partial list per column and head_topk_merge (the same kernel that closes the decode scan)
// picks the best k.
// blockIdx.x is the KV head: with 8 heads every XCD streams one head's keys through its L2.
//
// Measured on the 4096-row chunk of 4-head groups against 256 K keys (8.66 TFLOP, times of this
// kernel alone): the matrix instructions with nothing around them run at 1790 TFLOP/s on random
// operands (the chip's power limit, 0.72 of the 2.5 PFLOP/s peak: 4.8 ms); in this kernel's
// phase structure without any LDS read 5.2 ms, with the operand reads 6.3 ms, with the tile
// loads and the barrier 6.5 ms, with the filter and the lists 7.0 ms.  Other shapes tried, same
// work: one column block per wave (twice the operand reads per matrix instruction) 7.2 ms; one
// wave per SIMD with two column blocks 9.3 ms because nothing covers an insertion or the barrier;
// four column blocks per wave, or a second set of key operands, do not fit the register file
// of two waves per SIMD; key tiles that travel through registers (the compiler's count of loads
// in flight makes a step wait for the tile requested one step ago, not two) 7.9 ms.  The LDS
// itself is far from full: 128-bit reads with this pitch reach 205 B/clk per compute unit with 8
// waves (131 with 4), and the kernel asks for 64.
#include "common.hpp"

#include <type_traits>

namespace reattn {
namespace {

constexpr int kTileKeys = 128;
constexpr int kPitch = 272;                     // bytes per staged key row (256 + 16 pad)
constexpr int kBufs = 4;                        // staged key tiles (a power of two)
constexpr int kTileBytes = kTileKeys * kPitch;
constexpr int kFloorEvery = 16;                 // tiles between refreshes of the columns' shared floors (power of two)
constexpr int kFloorEach = 64, kFloorFourth = 512;   // ... every tile before the first, every fourth before the second

struct VoteGemmArgs {
  const uint16_t* k;        // key cache (bf16 bits)
  const uint16_t* q;        // [n_query][Hq][128] bf16 bits
  uint64_t* part;           // [n_query * Hq][n_split][KT] composites, best first
  int64_t ksh, kst, first_tok, n_keys;
  const int32_t* pt; int page_lg;   // paged cache (nullptr: none)
  int n_query, Hq, G, n_split, tiles_per_block;
};

__device__ __forceinline__ uint64_t vg_composite(float score, uint32_t pos) {
  return ((uint64_t)score_key(score) << 32) | (uint64_t)(0xffffffffu - pos);
}

// NCB: column blocks of 32 per wave; NW: waves of the workgroup (8: two per SIMD with half the register file each;
// 4: one per SIMD with all of it).  The workgroup owns NCB * 32 * NW columns; every wave walks all four key blocks
// of a tile for its own NCB column blocks.  The library launches NW = 8 with NCB = 2 (NCB = 1 for lists of 8, whose
// floor merge would not fit LDS, and for chunks of at most 2048 columns per KV head).
template <int KT, bool F16, int NCB, int NW>
__global__ __launch_bounds__(64 * NW) void vote_gemm_kernel(VoteGemmArgs a) {
  constexpr int kTileCols = NCB * 32 * NW;
  constexpr int kThreads = 64 * NW;
  static_assert(NW == 4 || NW == 8, "one or two waves per SIMD");
  static_assert((4 * NCB) % 2 == 0, "the accumulator sets alternate across tiles");
  typedef typename Mm<F16>::op8 op8;
  typedef mm_f32x16 f32x16;
  extern __shared__ __attribute__((aligned(16))) unsigned char vg_lds[];
  unsigned char* tiles = vg_lds;                            // kBufs staged key tiles, later the merge area

  const int tid = threadIdx.x, lane = tid & 63, cw = tid >> 6;
  const int ln = lane & 31, lh = lane >> 5;
  const int h = blockIdx.x;
  const int c0 = blockIdx.y * kTileCols;
  const int n_cols = a.n_query * a.G;                       // columns of this KV head: c = i * G + g
  const int64_t tile0 = (int64_t)blockIdx.z * a.tiles_per_block;
  const int64_t n_tiles_all = (a.n_keys + kTileKeys - 1) / kTileKeys;
  int64_t n_tiles = n_tiles_all - tile0;
  if (n_tiles > a.tiles_per_block) n_tiles = a.tiles_per_block;

  // query operands of this wave: NCB column blocks x 8 k-steps of 8 bf16 (columns past the end are zero)
  op8 bq[NCB][8];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const int c = c0 + (cw * NCB + cb) * 32 + ln;
    const bool live = c < n_cols;
    const int64_t qrow = live ? (int64_t)(c / a.G) * a.Hq + (int64_t)h * a.G + c % a.G : 0;
    const uint16_t* row = a.q + qrow * 128 + lh * 8;
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      u32x4 w = *(const u32x4*)(row + ks * 16);
      if (!live) w = u32x4{0u, 0u, 0u, 0u};
      bq[cb][ks] = __builtin_bit_cast(op8, w);
      // the query operands stay in the accumulation half of the register file (a matrix instruction reads
      // either half), which leaves the other half to the scores and the key tiles in flight
      if (NW == 4) asm volatile("" : "+a"(bq[cb][ks]));
    }
  }
  // running lists: KT best (score, key) pairs of each of this lane's NCB columns over the keys this lane has
  // seen, best first, in registers; lv[cb][KT - 1] is the bar a new score has to clear
  float lv[NCB][KT];
  uint32_t li[NCB][KT];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
    for (int y = 0; y < KT; ++y) { lv[cb][y] = -__builtin_inff(); li[cb][y] = 0xffffffffu; }
  // A column has two partial lists (the lane halves).  Every kFloorEvery tiles (more often early on) the lists' scores meet in LDS
  // (lvx), one thread per column merges them and publishes the column's true k-th value so far (`floor`):
  // a score below it cannot end among the column's k best, so each list admits about half of what it would
  // on its own.  A score equal to the floor may still win on its lower key, so it passes.
  float* lvx = (float*)(vg_lds + kBufs * kTileBytes);       // [NCB * KT][kThreads]
  float* xfloor = lvx + NCB * KT * kThreads;                // [kTileCols]
  for (int c = tid; c < kTileCols; c += kThreads) xfloor[c] = -__builtin_inff();

  // staging: key tiles travel from memory straight into LDS (global_load_lds_dwordx4: lane L of a wave puts its
  // 16 bytes at m0 + 16 L, no register in between), three tiles ahead of the matrix work: step t requests tile
  // t + 3 into the buffer tile t - 1 has left, and the barrier that ends step t + 1 is the first that needs it
  // (two steps of slack: a step is under 2 us, a trip to memory under load is not always).  A tile is 128 rows
  // of 17 slots of 16 bytes (16 pieces of the row + one pad: the 272-byte pitch keeps the operand reads of 32
  // rows off each other's banks); the pad slot receives a copy of the last piece.  Its 2176 slots are 34 wave
  // loads of 64; wave w of W issues loads W i + w, i < 32 / W, and, so that every wave counts the same number of loads in
  // flight per tile, load 32 + (w & 1): the two loads issued twice write the same bytes twice.
  constexpr int kDmaEach = 32 / NW, kDma = kDmaEach + 1;
  const int64_t row_bytes = a.kst * 2;
  const char* khead = (const char*)(a.k + (int64_t)h * a.ksh);
  const char* kmid = khead + a.first_tok * row_bytes;
  uint32_t voff[kDma];                                      // row * row_bytes + piece * 16 of this lane's slot of load i
#pragma unroll
  for (int i = 0; i < kDma; ++i) {
    const int slot = (i < kDmaEach ? i * NW + cw : 32 + (cw & 1)) * 64 + lane;
    const int row = slot / 17, piece = slot % 17;
    voff[i] = (uint32_t)(row * row_bytes) + (uint32_t)(piece < 16 ? piece : 15) * 16u;
  }
  const uint32_t lds_tiles = (uint32_t)(uintptr_t)tiles;
  auto dma_dst = [&](int buf, int i) -> uint32_t {           // LDS byte address of load i of this wave (wave-uniform)
    return (uint32_t)__builtin_amdgcn_readfirstlane((int)(lds_tiles + (uint32_t)buf * kTileBytes + (uint32_t)(i < kDmaEach ? i * NW + cw : 32 + (cw & 1)) * 1024u));
  };
  // whole: every row of the tile exists (a compile-time yes skips the question).  Through a page table a tile of
  // 128 consecutive tokens lies in at most three pages (pages hold 64 tokens or more): their first rows are read
  // with scalar loads, which the counter of the tile loads does not see, and a lane picks one by its token's page.
  auto dma_tile = [&](auto whole, int64_t tile, int buf) __attribute__((always_inline)) {
    if (!a.pt && (decltype(whole)::value || (tile + 1) * kTileKeys <= a.n_keys)) {
      const char* base = kmid + tile * kTileKeys * row_bytes;      // workgroup-uniform
#pragma unroll
      for (int i = 0; i < kDma; ++i)
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, %2"
                     :: "s"(dma_dst(buf, i)), "v"(voff[i]), "s"(base) : "memory");
    } else {                                                 // through the page table, or a ragged last tile
      const int64_t tok0 = a.first_tok + tile * kTileKeys, tok_last = a.first_tok + a.n_keys - 1;
      int64_t pg[3] = {0, 0, 0};
      int64_t pg0 = 0;
      if (a.pt) {
        pg0 = tok0 >> a.page_lg;
        const int64_t pg_last = tok_last >> a.page_lg;
        // workgroup-uniform, and read as constant memory so that the loads are scalar ones (the kernel never writes the table)
        typedef const __attribute__((address_space(4))) int32_t* const_i32;
        const const_i32 pt = (const_i32)(uintptr_t)a.pt;
#pragma unroll
        for (int i = 0; i < 3; ++i) pg[i] = (int64_t)pt[pg0 + i < pg_last ? pg0 + i : pg_last] << a.page_lg;
      }
#pragma unroll
      for (int i = 0; i < kDma; ++i) {
        const int slot = (i < kDmaEach ? i * NW + cw : 32 + (cw & 1)) * 64 + lane;
        const int row = slot / 17, piece = slot % 17;
        int64_t tok = tok0 + row;
        if (tok > tok_last) tok = tok_last;                  // rows past the end repeat the last key; their scores are dropped
        int64_t mrow = tok;
        if (a.pt) {
          const int64_t d = (tok >> a.page_lg) - pg0;
          mrow = (d == 0 ? pg[0] : d == 1 ? pg[1] : pg[2]) | (tok & (((int64_t)1 << a.page_lg) - 1));
        }
        const char* src = khead + mrow * row_bytes + (piece < 16 ? piece : 15) * 16;
        asm volatile("s_mov_b32 m0, %0\n\ts_nop 0\n\tglobal_load_lds_dwordx4 %1, off"
                     :: "s"(dma_dst(buf, i)), "v"(src) : "memory");
      }
    }
  };
  constexpr std::true_type yes{};
  constexpr std::false_type no{};
  for (int i = 0; i < 3 && i < n_tiles; ++i) dma_tile(no, tile0 + i, i);
  asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
  __syncthreads();

  // C layout of a 32x32 block: acc[i] is key row (i/4)*8 + (lane/32)*4 + i%4, column lane%32.
  f32x16 accs[2];                                           // one in the matrix pipe, one under the filter
  op8 av[8];
  auto rows_of = [&](int buf, int j) -> const unsigned char* {
    return tiles + buf * kTileBytes + (j * 32 + ln) * kPitch + lh * 16;
  };
  // acc <- keys in av x queries of column block cb; av <- the rows at `refill` (refills: a compile-time yes or no)
  auto contract = [&](f32x16& acc, int cb, auto refills, const unsigned char* refill) __attribute__((always_inline)) {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) {
      if (ks == 0) {
        f32x16 z;
#pragma unroll
        for (int i = 0; i < 16; ++i) z[i] = 0.f;
        acc = Mm<F16>::mfma32(av[0], bq[cb][0], z);
      } else {
        acc = Mm<F16>::mfma32(av[ks], bq[cb][ks], acc);
      }
      if (decltype(refills)::value) av[ks] = *(const op8*)(refill + ks * 32);
    }
    // the matrix instructions are issued here, ahead of the filter that follows in program order, and their
    // results live in the registers the vector unit reads
    asm volatile("" : "+v"(acc));
  };
  float floor_[NCB];
  // the scores of one key block of column block cb against the running list; key_blk: key of acc[0] of this lane
  auto filter = [&](auto ragged, f32x16& acc, int cb, int64_t key_blk) __attribute__((always_inline)) {
    if (decltype(ragged)::value) {                          // only a ragged last tile: keys past the end never enter a list
#pragma unroll
      for (int i = 0; i < 16; ++i)
        if (key_blk + (i >> 2) * 8 + (i & 3) >= a.n_keys) acc[i] = -__builtin_inff();
    }
    float m = acc[0];
#pragma unroll
    for (int i = 1; i < 16; ++i) m = fmaxf(m, acc[i]);
    // A score enters a list rarely (the list's k-th value climbs quickly), and then usually one per lane: take
    // the lane's largest remaining score, insert, strike it out, again.  Largest first and, among equals,
    // lowest key first: an equal score never displaces.
    while (__any(m > lv[cb][KT - 1] && m >= floor_[cb])) {
      if (m > lv[cb][KT - 1] && m >= floor_[cb]) {
        int at = 15;
#pragma unroll
        for (int i = 14; i >= 0; --i) at = acc[i] == m ? i : at;             // lowest i holding the maximum
        const uint32_t key = (uint32_t)(key_blk + (at >> 2) * 8 + (at & 3));
        // entries at least as large stay above the new one (their keys are lower)
        bool above[KT];
#pragma unroll
        for (int y = 0; y < KT; ++y) above[y] = lv[cb][y] >= m;
#pragma unroll
        for (int y = KT - 1; y >= 0; --y) {
          const bool here = y == 0 || above[y - 1];           // the new entry lands at y or above
          lv[cb][y] = above[y] ? lv[cb][y] : here ? m : lv[cb][y - 1];
          li[cb][y] = above[y] ? li[cb][y] : here ? key : li[cb][y - 1];
        }
        float mm = -__builtin_inff();
#pragma unroll
        for (int i = 0; i < 16; ++i) {
          acc[i] = i == at ? -__builtin_inff() : acc[i];
          mm = fmaxf(mm, acc[i]);
        }
        m = mm;
      }
    }
  };

  // One tile.
  // bc: buffer of tile t.  `full`: tiles t + 1 .. t + 3 all exist and are whole, so the step has no branch but
  // the rare insertions (and the one on the page table) and waits only for the tile due.
  auto step = [&](auto ragged, auto full, int64_t t, int bc) __attribute__((always_inline)) {
    constexpr bool kFull = decltype(full)::value;
    const int bn = (bc + 1) & (kBufs - 1);                  // buffer of tile t + 1
    const int bd = (bc + 3) & (kBufs - 1);                  // buffer of tile t + 3: tile t - 1 has left it
    const bool more = kFull || t + 1 < n_tiles;
    const int64_t key0 = (tile0 + t) * kTileKeys + lh * 4;
    // Phase q = (key block j, column block cb) of the tile, j-major.  On entry phase 0 is in the matrix pipe
    // and av holds the rows of block 0 (of block 1 if there is one column block: the last column block of a key
    // block refills av behind its matrix instructions).  Each turn issues the matrix work of phase q + 1, then
    // filters phase q.
#pragma unroll
    for (int q = 0; q < 4 * NCB; ++q) {
      const int j = q / NCB, cb = q % NCB;
      const int jn = (q + 1) / NCB, cbn = (q + 1) % NCB;    // jn == 4: the first block of tile t + 1
      const bool last_cb = cbn == NCB - 1;
      if (jn < 4) {
        // rows after block jn: of this tile, or the first of the next
        if (last_cb && jn < 3) contract(accs[(q + 1) & 1], cbn, yes, rows_of(bc, jn + 1));
        else if (last_cb && more) contract(accs[(q + 1) & 1], cbn, yes, rows_of(bn, 0));
        else contract(accs[(q + 1) & 1], cbn, no, nullptr);
      } else if (more) {
        if (last_cb) contract(accs[(q + 1) & 1], cbn, yes, rows_of(bn, 1));
        else contract(accs[(q + 1) & 1], cbn, no, nullptr);
      }
      if (q == 0) {
        if (kFull || t + 3 < n_tiles) dma_tile(full, tile0 + t + 3, bd);
#pragma unroll
        for (int x = 0; x < NCB; ++x) floor_[x] = xfloor[(cw * NCB + x) * 32 + ln];
      }
      filter(ragged, accs[q & 1], cb, key0 + j * 32);
    }
    // workgroup-uniform.  Early in the walk the lists move with every block and a fresh floor keeps half of the
    // scores that would enter one of them out: refreshes are dense there (1.7 ms of filter work became 0.7).
    if ((t & (kFloorEvery - 1)) == kFloorEvery - 1 || t < kFloorEach || (t < kFloorFourth && (t & 3) == 3)) {
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb)
#pragma unroll
        for (int y = 0; y < KT; ++y) lvx[(cb * KT + y) * kThreads + tid] = lv[cb][y];
      __syncthreads();
      for (int col = tid; col < kTileCols; col += kThreads) {
        // column col = cw2 * 32 + ln: its lists sit with lanes {0, 32} + ln of wave cw2 / NCB, block cw2 % NCB
        const int cw2 = col >> 5, lcol = col & 31, ccw = cw2 / NCB, ccb = cw2 % NCB;
        float best[KT];
#pragma unroll
        for (int y = 0; y < KT; ++y) best[y] = -__builtin_inff();
#pragma unroll
        for (int part = 0; part < 2; ++part) {
          const int owner = ccw * 64 + part * 32 + lcol;
#pragma unroll
          for (int y = 0; y < KT; ++y) {
            float v = lvx[(ccb * KT + y) * kThreads + owner];
#pragma unroll
            for (int z = 0; z < KT; ++z) {                  // keep the KT largest, descending
              const float hi = fmaxf(best[z], v);
              v = fminf(best[z], v);
              best[z] = hi;
            }
          }
        }
        xfloor[col] = best[KT - 1];
      }
    }
    // tile t + 2 has landed (requested during step t - 1); the loads of this step may still fly
    if (kFull) asm volatile("s_waitcnt vmcnt(%0)" :: "n"(kDma) : "memory");
    else asm volatile("s_waitcnt vmcnt(0)" ::: "memory");
    __syncthreads();
  };

  if (n_tiles > 0) {
#pragma unroll
    for (int ks = 0; ks < 8; ++ks) av[ks] = *(const op8*)(rows_of(0, 0) + ks * 32);
    if (NCB == 1) contract(accs[0], 0, yes, rows_of(0, 1));
    else contract(accs[0], 0, no, nullptr);
  }
  const bool ragged_last = tile0 + n_tiles == n_tiles_all && (a.n_keys % kTileKeys) != 0;
  int bc = 0;
  int64_t t = 0;
  // the long middle of the walk: a loop of its own with a single path through it
  for (; t + 3 < n_tiles; ++t) {
    step(no, yes, t, bc);
    bc = (bc + 1) & (kBufs - 1);
  }
  for (; t < n_tiles; ++t) {
    if (ragged_last && t == n_tiles - 1) step(yes, no, t, bc);
    else step(no, no, t, bc);
    bc = (bc + 1) & (kBufs - 1);
  }

  // the two partial lists of a column (the lane halves) meet in LDS (over the key tiles)
  constexpr int P = 2;
  uint64_t* lists = (uint64_t*)vg_lds;                      // [kTileCols][P][KT]
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const int col = (cw * NCB + cb) * 32 + ln;
#pragma unroll
    for (int y = 0; y < KT; ++y)
      lists[((size_t)col * P + lh) * KT + y] = li[cb][y] != 0xffffffffu ? vg_composite(lv[cb][y], li[cb][y]) : 0ull;
  }
  __syncthreads();
  for (int col = tid; col < kTileCols && c0 + col < n_cols; col += kThreads) {
    const int c = c0 + col;
    const uint64_t* mine = lists + (size_t)col * P * KT;
    int head[P];
#pragma unroll
    for (int x = 0; x < P; ++x) head[x] = 0;
    uint64_t* out = a.part + (((int64_t)(c / a.G) * a.Hq + (int64_t)h * a.G + c % a.G) * a.n_split + blockIdx.z) * KT;
    for (int round = 0; round < KT; ++round) {              // lists are sorted: compare their heads
      uint64_t best = 0ull; int from = 0;
#pragma unroll
      for (int x = 0; x < P; ++x) {
        const uint64_t v = head[x] < KT ? mine[x * KT + head[x]] : 0ull;
        if (v > best) { best = v; from = x; }
      }
#pragma unroll
      for (int x = 0; x < P; ++x) head[x] += (x == from && best != 0ull) ? 1 : 0;
      out[round] = best;
    }
  }
}

template <int KT, bool F16, int NCB, int NW>
hipError_t vote_gemm_launch(const VoteGemmArgs& a, dim3 grid, hipStream_t st) {
  constexpr int kTileCols = NCB * 32 * NW, kThreads = 64 * NW;
  static_assert((size_t)kTileCols * 2 * KT * sizeof(uint64_t) <= kBufs * (size_t)kTileBytes, "merge area inside the tiles");
  constexpr size_t lds = kBufs * (size_t)kTileBytes + (size_t)NCB * KT * kThreads * 4 + kTileCols * 4;
  static_assert(lds <= (size_t)160 * 1024, "fits a compute unit's LDS");
  auto kern = vote_gemm_kernel<KT, F16, NCB, NW>;
  hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, grid, dim3(kThreads), lds, st, a);
  return hipGetLastError();
}

}  // namespace

// Columns per workgroup: 512 (two column blocks per wave) where the lists are short and the chunk has more than
// 2048 columns per KV head; below that the keys are split eight ways to fill the chip and the longer key runs
// of 256-column workgroups win (512 rows of 4-head groups against 256 K keys: 1.15 against 1.28 ms).
int vote_gemm_tile_cols(const Plan& pl, int n_query, int list_len) {
  return list_len <= 4 && (int64_t)n_query * pl.G > 2048 ? 512 : 256;
}

// Key splits of the chunk contraction: enough workgroups for one round over the chip (one workgroup per CU: a
// second round only repeats the insertion-heavy start of every running list).
static int gemm_splits(const Plan& pl, int n_query, int tile_cols) {
  const int64_t col_tiles = ((int64_t)n_query * pl.G + tile_cols - 1) / tile_cols;
  const int64_t n_tiles = (pl.n_mid + kTileKeys - 1) / kTileKeys;
  int64_t split = (256 + col_tiles * pl.Hkv - 1) / (col_tiles * pl.Hkv);
  if (split > n_tiles) split = n_tiles;
  if (split < 1) split = 1;
  const int64_t per = (n_tiles + split - 1) / split;        // tiles per workgroup
  return (int)((n_tiles + per - 1) / per);
}
int vote_gemm_splits(const Plan& pl, int n_query, int list_len) {
  return gemm_splits(pl, n_query, vote_gemm_tile_cols(pl, n_query, list_len));
}

// part: [n_query * Hq][splits][list_len] composites (list_len = vote_list_len(vote_k)).
hipError_t launch_vote_gemm(const Plan& pl, const void* q, int n_query, const void* k_cache, int list_len,
                            uint64_t* part, hipStream_t st) {
  if (n_query <= 0 || pl.n_mid <= 0) return hipSuccess;
  VoteGemmArgs a;
  a.k = (const uint16_t*)k_cache; a.q = (const uint16_t*)q; a.part = part;
  a.ksh = pl.ksh; a.kst = pl.kst; a.first_tok = pl.s_eff; a.n_keys = pl.n_mid; a.pt = pl.pt; a.page_lg = pl.page_lg;
  a.n_query = n_query; a.Hq = pl.Hq; a.G = pl.G;
  const int tile_cols = vote_gemm_tile_cols(pl, n_query, list_len);
  a.n_split = gemm_splits(pl, n_query, tile_cols);
  const int64_t n_tiles = (pl.n_mid + kTileKeys - 1) / kTileKeys;
  a.tiles_per_block = (int)((n_tiles + a.n_split - 1) / a.n_split);
  const dim3 grid((unsigned)pl.Hkv, (unsigned)(((int64_t)n_query * pl.G + tile_cols - 1) / tile_cols),
                  (unsigned)a.n_split);
  if (pl.dtype == kF16) {
    switch (list_len) {
      case 1: return (tile_cols == 512 ? vote_gemm_launch<1, true, 2, 8>(a, grid, st) : vote_gemm_launch<1, true, 1, 8>(a, grid, st));
      case 2: return (tile_cols == 512 ? vote_gemm_launch<2, true, 2, 8>(a, grid, st) : vote_gemm_launch<2, true, 1, 8>(a, grid, st));
      case 4: return (tile_cols == 512 ? vote_gemm_launch<4, true, 2, 8>(a, grid, st) : vote_gemm_launch<4, true, 1, 8>(a, grid, st));
      default: return vote_gemm_launch<8, true, 1, 8>(a, grid, st);
    }
  }
  switch (list_len) {
    case 1: return (tile_cols == 512 ? vote_gemm_launch<1, false, 2, 8>(a, grid, st) : vote_gemm_launch<1, false, 1, 8>(a, grid, st));
    case 2: return (tile_cols == 512 ? vote_gemm_launch<2, false, 2, 8>(a, grid, st) : vote_gemm_launch<2, false, 1, 8>(a, grid, st));
    case 4: return (tile_cols == 512 ? vote_gemm_launch<4, false, 2, 8>(a, grid, st) : vote_gemm_launch<4, false, 1, 8>(a, grid, st));
    default: return vote_gemm_launch<8, false, 1, 8>(a, grid, st);
  }
}

}  // namespace reattn
