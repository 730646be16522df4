// Vote selection for a chunk of query rows: the per-head top-k lists of every (query row,
// query head) (paper, Method, "Full-Context Cache Selection", last paragraph: each head and
// each query votes with its own top-k) against the whole middle of the key cache are one
// dense contraction per KV head, [M * G columns] x [N_mid keys] x [D], so it runs on the
// matrix cores (v_mfma_f32_32x32x16_bf16, fp32 accumulation) with the top-k fused behind it:
// no score is ever written.  bf16 storage makes every head's query an exact MFMA operand, so
// unlike the group-sum contraction there is no hi/lo split and the executed matrix work
// equals the algorithmic 2 * M * Hq * N_mid * D.
//
// Tiling: a workgroup of 8 waves owns 256 columns ((query row, head) pairs, query-major) of
// one KV head and walks key tiles of 128 rows staged through LDS (two buffers, 272-byte row
// pitch, the tile after next travelling through registers).  Keys are the A operand, so a
// lane of a 32x32 block holds ONE column and 16 keys: the running top-k list of a column
// belongs to the lane that owns it (the list in LDS, its k-th value in a register), and a
// tile costs a maximum over 16 scores and one comparison unless a score enters the list.
// Wave (kw, cw) takes the key blocks 2kw, 2kw + 1 of the tile and the two column blocks of
// quarter cw (their 2 x 8 query operands, 64 VGPRs, stay in registers).  The four partial
// lists of a column (2 wave rows x 2 lane halves) are merged through LDS
// at the end.  With few query rows the keys are also split over blockIdx.z so that the chip
// is filled; every workgroup writes one partial list per column and head_topk_merge (the
// same kernel that closes the decode scan) picks the best k.
// blockIdx.x is the KV head: with 8 heads every XCD streams one head's keys through its L2.
#include "common.hpp"

namespace reattn {
namespace {

typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x16 __attribute__((ext_vector_type(16)));

constexpr int kTileKeys = 128;
constexpr int kPitch = 272;                     // bytes per staged key row (256 + 16 pad)
constexpr int kThreads = 512;                   // 8 waves: 2 pairs of key blocks x 4 column quarters
constexpr int kColBlocksMax = 4;                // column blocks of 32 a wave may own (2 or 4: 256 or 512 columns per workgroup)
constexpr int kTileBytes = kTileKeys * kPitch;
constexpr int kStageNS = 2048 / kThreads;       // 16-byte pieces of a key tile per thread
constexpr int kFloorEvery = 32;                 // tiles between refreshes of the columns' shared floors (power of two)

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

// NCB: column blocks of 32 per wave; the workgroup owns NCB * 128 columns.  With NCB = 4 a key operand read from
// LDS feeds four matrix instructions instead of two, the barrier and the staging of a tile are spread over twice
// the matrix work, and the 64 column tiles of config 4's chunk become 32 per KV head: one round of workgroups per
// chiplet, so the keys enter the chip once instead of twice.
template <int KT, bool F16, int NCB>
__global__ __launch_bounds__(kThreads) void vote_gemm_kernel(VoteGemmArgs a) {
  constexpr int kTileCols = NCB * 128;
  typedef typename Mm<F16>::op8 op8;
  extern __shared__ __attribute__((aligned(16))) unsigned char vg_lds[];
  unsigned char* tiles = vg_lds;                            // two staged key tiles, later the merge area

  const int tid = threadIdx.x, lane = tid & 63, wave = tid >> 6;
  const int kw = wave & 1, cw = wave >> 1;
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
    }
  }
  // running lists: entry t of column block cb of this thread at lv/li[(cb * KT + t) * kThreads + tid]
  // (best first); only the k-th value, the bar a new score has to clear, lives in a register
  float* lv = (float*)(vg_lds + 2 * kTileBytes);
  uint32_t* li = (uint32_t*)(lv + NCB * KT * kThreads);
  // A column has four partial lists (2 wave rows x 2 lane halves).  Every kFloorEvery tiles one thread
  // per column merges them and publishes the column's true k-th value so far (`floor`): a score below
  // it cannot end among the column's k best, so each list admits about a quarter of what it would on
  // its own.  A score equal to the floor may still win on its lower key, so it passes.
  float* xfloor = (float*)(li + NCB * KT * kThreads);       // [kTileCols]
  for (int c = tid; c < kTileCols; c += kThreads) xfloor[c] = -__builtin_inff();
  float bar[NCB];
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    bar[cb] = -__builtin_inff();
#pragma unroll
    for (int t = 0; t < KT; ++t) { lv[(cb * KT + t) * kThreads + tid] = -__builtin_inff(); li[(cb * KT + t) * kThreads + tid] = 0xffffffffu; }
  }

  // staging: thread t moves kStageNS x 16 bytes of the 128 x 256-byte key tile (rows t/16 + 32j,
  // piece t%16); tile t + 2 is requested right after tile t + 1 went from the same registers to LDS
  constexpr int RS = kThreads / 16;
  const int srow = tid >> 4, scol = tid & 15;
  const int64_t row_bytes = a.kst * 2;
  const char* kbase = (const char*)(a.k + (int64_t)h * a.ksh + a.first_tok * a.kst) + scol * 16;
  const char* next = kbase + (tile0 * kTileKeys + srow) * row_bytes;
  u32x4 stg[kStageNS];
  auto load_tile = [&](int64_t tile, u32x4* s) {
    if (a.pt) {                                              // paged cache: every row through the page table
      const char* hbase = (const char*)(a.k + (int64_t)h * a.ksh) + scol * 16;
#pragma unroll
      for (int j = 0; j < kStageNS; ++j) {
        int64_t key = tile * kTileKeys + srow + RS * j;
        if (key >= a.n_keys) key = a.n_keys - 1;
        s[j] = *(const u32x4*)(hbase + paged_row(a.pt, a.page_lg, a.first_tok + key) * row_bytes);
      }
    } else if ((tile + 1) * kTileKeys <= a.n_keys) {         // every tile but a ragged last one
#pragma unroll
      for (int j = 0; j < kStageNS; ++j) s[j] = *(const u32x4*)(next + (int64_t)(RS * j) * row_bytes);
    } else {
#pragma unroll
      for (int j = 0; j < kStageNS; ++j) {
        int64_t key = tile * kTileKeys + srow + RS * j;
        if (key >= a.n_keys) key = a.n_keys - 1;             // rows past the end repeat the last key; their scores are dropped
        s[j] = *(const u32x4*)(kbase + key * row_bytes);
      }
    }
    next += (int64_t)kTileKeys * row_bytes;
  };
  auto stash_tile = [&](int buf, const u32x4* s) {
#pragma unroll
    for (int j = 0; j < kStageNS; ++j)
      *(u32x4*)(tiles + buf * kTileBytes + (srow + RS * j) * kPitch + scol * 16) = s[j];
  };

  // Tile t + 1 is written to LDS during step t from registers that were loaded during step t - 2: two steps of
  // slack (a step is under 2 us, a trip to HBM under load is not always).  Two register sets, by tile parity.
  u32x4 stg2[kStageNS];
  if (n_tiles > 0) {
    load_tile(tile0, stg);
    stash_tile(0, stg);
    if (n_tiles > 1) load_tile(tile0 + 1, stg2);             // odd tiles travel in stg2
    if (n_tiles > 2) load_tile(tile0 + 2, stg);              // even tiles in stg
  }
  __syncthreads();

  // C layout of a 32x32 block: acc[i] is key row (i/4)*8 + (lane/32)*4 + i%4, column lane%32.
  // The two waves of a SIMD (waves w and w + 4) move the next tile into LDS at opposite ends of a step, so that
  // one of them always has matrix work in flight while the other writes.
  const bool stash_first = (wave >> 2) == 0;
  auto step = [&](int64_t t, int buf, u32x4* s) {            // s: the registers that hold tile t + 1
    if (stash_first) {
      if (t + 1 < n_tiles) stash_tile(buf ^ 1, s);
      if (t + 3 < n_tiles) load_tile(tile0 + t + 3, s);
    }
    float floor_[NCB];
#pragma unroll
    for (int cb = 0; cb < NCB; ++cb) floor_[cb] = xfloor[(cw * NCB + cb) * 32 + ln];
#pragma unroll
    for (int j = 0; j < 2; ++j) {                           // the two key blocks of this wave
      const int kb = kw * 2 + j;
      const unsigned char* arow = tiles + buf * kTileBytes + (kb * 32 + ln) * kPitch + lh * 16;
      const int64_t key_blk = (tile0 + t) * kTileKeys + kb * 32 + lh * 4;
      f32x16 acc[NCB];
#pragma unroll
      for (int x = 0; x < NCB; ++x)
#pragma unroll
        for (int i = 0; i < 16; ++i) acc[x][i] = 0.f;
#pragma unroll
      for (int ks = 0; ks < 8; ++ks) {
        const op8 av = *(const op8*)(arow + ks * 32);
#pragma unroll
        for (int x = 0; x < NCB; ++x) acc[x] = Mm<F16>::mfma32(av, bq[x][ks], acc[x]);
      }
      if (key_blk + 27 >= a.n_keys) {                       // only the last tile: keys past the end never enter a list
#pragma unroll
        for (int x = 0; x < NCB; ++x)
#pragma unroll
          for (int i = 0; i < 16; ++i)
            if (key_blk + (i >> 2) * 8 + (i & 3) >= a.n_keys) acc[x][i] = -__builtin_inff();
      }
#pragma unroll
      for (int cb = 0; cb < NCB; ++cb) {
        float m = acc[cb][0];
#pragma unroll
        for (int i = 1; i < 16; ++i) m = fmaxf(m, acc[cb][i]);
        // A score enters a list rarely (the list's k-th value climbs quickly), and then usually
        // one per lane: take the lane's largest remaining score, insert, strike it out, again.
        // Largest first and, among equals, lowest key first: an equal score never displaces.
        while (__any(m > bar[cb] && m >= floor_[cb])) {
          if (m > bar[cb] && m >= floor_[cb]) {
            int at = 15;
#pragma unroll
            for (int i = 14; i >= 0; --i) at = acc[cb][i] == m ? i : at;     // lowest i holding the maximum
            float v[KT]; uint32_t id[KT];
#pragma unroll
            for (int y = 0; y < KT - 1; ++y) { v[y] = lv[(cb * KT + y) * kThreads + tid]; id[y] = li[(cb * KT + y) * kThreads + tid]; }
            v[KT - 1] = m; id[KT - 1] = (uint32_t)(key_blk + (at >> 2) * 8 + (at & 3));
#pragma unroll
            for (int y = KT - 1; y > 0; --y) {
              if (v[y] > v[y - 1]) {
                const float fv = v[y]; v[y] = v[y - 1]; v[y - 1] = fv;
                const uint32_t iv = id[y]; id[y] = id[y - 1]; id[y - 1] = iv;
              }
            }
#pragma unroll
            for (int y = 0; y < KT; ++y) { lv[(cb * KT + y) * kThreads + tid] = v[y]; li[(cb * KT + y) * kThreads + tid] = id[y]; }
            bar[cb] = v[KT - 1];
            m = -__builtin_inff();
#pragma unroll
            for (int i = 0; i < 16; ++i) {
              acc[cb][i] = i == at ? -__builtin_inff() : acc[cb][i];
              m = fmaxf(m, acc[cb][i]);
            }
          }
        }
      }
    }
    if (!stash_first) {
      if (t + 1 < n_tiles) stash_tile(buf ^ 1, s);
      if (t + 3 < n_tiles) load_tile(tile0 + t + 3, s);
    }
    if ((t & (kFloorEvery - 1)) == kFloorEvery - 1) {       // workgroup-uniform
      __syncthreads();                                      // every list is at rest
      for (int col = tid; col < kTileCols; col += kThreads) {
        // column col = (cw2 * 32 + ln): its lists sit with threads (cw * 2 + kw) * 64 + lh * 32 + ln
        const int cw2 = col >> 5, lcol = col & 31, ccw = cw2 / NCB, ccb = cw2 % NCB;
        float best[KT];
#pragma unroll
        for (int y = 0; y < KT; ++y) best[y] = -__builtin_inff();
#pragma unroll
        for (int part = 0; part < 4; ++part) {
          const int owner = (ccw * 2 + (part >> 1)) * 64 + (part & 1) * 32 + lcol;
#pragma unroll
          for (int y = 0; y < KT; ++y) {
            float v = lv[(ccb * KT + y) * kThreads + owner];
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
    __syncthreads();
  };

  for (int64_t t = 0; t < n_tiles; t += 2) {
    step(t, 0, stg2);
    if (t + 1 < n_tiles) step(t + 1, 1, stg);
  }

  // the four partial lists of a column (2 wave rows x 2 lane halves) meet in LDS (over the key tiles)
  uint64_t* lists = (uint64_t*)vg_lds;                      // [kTileCols][4][KT]
#pragma unroll
  for (int cb = 0; cb < NCB; ++cb) {
    const int col = (cw * NCB + cb) * 32 + ln;
#pragma unroll
    for (int t = 0; t < KT; ++t) {
      const float v = lv[(cb * KT + t) * kThreads + tid];
      const uint32_t id = li[(cb * KT + t) * kThreads + tid];
      lists[((size_t)col * 4 + kw * 2 + lh) * KT + t] = id != 0xffffffffu ? vg_composite(v, id) : 0ull;
    }
  }
  __syncthreads();
  for (int col = tid; col < kTileCols && c0 + col < n_cols; col += kThreads) {
    const int c = c0 + col;
    const uint64_t* mine = lists + (size_t)col * 4 * KT;
    int head[4];
#pragma unroll
    for (int s = 0; s < 4; ++s) head[s] = 0;
    uint64_t* out = a.part + (((int64_t)(c / a.G) * a.Hq + (int64_t)h * a.G + c % a.G) * a.n_split + blockIdx.z) * KT;
    for (int round = 0; round < KT; ++round) {              // lists are sorted: compare their heads
      uint64_t best = 0ull; int from = 0;
#pragma unroll
      for (int s = 0; s < 4; ++s) {
        const uint64_t v = head[s] < KT ? mine[s * KT + head[s]] : 0ull;
        if (v > best) { best = v; from = s; }
      }
#pragma unroll
      for (int s = 0; s < 4; ++s) head[s] += (s == from && best != 0ull) ? 1 : 0;
      out[round] = best;
    }
  }
}

template <int KT, bool F16, int NCB>
hipError_t vote_gemm_launch(const VoteGemmArgs& a, dim3 grid, hipStream_t st) {
  constexpr int kTileCols = NCB * 128;
  static_assert((size_t)kTileCols * 4 * KT * sizeof(uint64_t) <= 2 * (size_t)kTileBytes, "merge area inside the tiles");
  constexpr size_t lds = 2 * (size_t)kTileBytes + (size_t)NCB * KT * kThreads * 8 + kTileCols * 4;
  static_assert(lds <= (size_t)160 * 1024, "fits a compute unit's LDS");
  auto kern = vote_gemm_kernel<KT, F16, NCB>;
  hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, grid, dim3(kThreads), lds, st, a);
  return hipGetLastError();
}

}  // namespace

// Columns per workgroup: 512 while the lists of a column block fit LDS four times over (lists of up to 4) and the
// chunk has columns to fill them, else 256.
int vote_gemm_tile_cols(const Plan& pl, int n_query, int list_len) {
  (void)pl; (void)n_query; (void)list_len;
  return 256;
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
  const bool wide = tile_cols == 512;
  if (pl.dtype == kF16) {
    switch (list_len) {
      case 1: return wide ? vote_gemm_launch<1, true, 4>(a, grid, st) : vote_gemm_launch<1, true, 2>(a, grid, st);
      case 2: return wide ? vote_gemm_launch<2, true, 4>(a, grid, st) : vote_gemm_launch<2, true, 2>(a, grid, st);
      case 4: return wide ? vote_gemm_launch<4, true, 4>(a, grid, st) : vote_gemm_launch<4, true, 2>(a, grid, st);
      default: return vote_gemm_launch<8, true, 2>(a, grid, st);
    }
  }
  switch (list_len) {
    case 1: return wide ? vote_gemm_launch<1, false, 4>(a, grid, st) : vote_gemm_launch<1, false, 2>(a, grid, st);
    case 2: return wide ? vote_gemm_launch<2, false, 4>(a, grid, st) : vote_gemm_launch<2, false, 2>(a, grid, st);
    case 4: return wide ? vote_gemm_launch<4, false, 4>(a, grid, st) : vote_gemm_launch<4, false, 2>(a, grid, st);
    default: return vote_gemm_launch<8, false, 2>(a, grid, st);
  }
}

}  // namespace reattn
