// Vote selection (paper, Method, "Full-Context Cache Selection", last paragraph; Setup:
// k = 4, k' = 127, span 32): every (query row, query head) votes for its own top-k middle
// tokens by raw position-agnostic score, the k' most voted tokens are kept together with
// their m neighbouring entries, overlaps deduplicated; one shared set per layer.
//
//   head_topk_scan   the fused score + top-k of the paper: the key cache is streamed once with
//                    16-byte non-temporal loads and every lane keeps a running top-k in
//                    registers, so no score ever leaves the chip.  bf16 / D = 128 scores on the
//                    matrix cores (head_topk_mfma_kernel: up to 32 (query row, head) columns
//                    per pass over the keys); fp32 / D = 64 on the vector ALU with DPP row
//                    reductions (head_topk_scan_kernel, one pass per query row).  Lists are
//                    merged inside the wave, then over the waves, and each workgroup writes k
//                    (score, index) composites per (query row, head);
//   head_topk_merge  one wave per (query, head): the best k of the workgroups' partial lists,
//                    ascending absolute indices;
//   vote_merge_small up to 1024 votes (a decode step): one workgroup counts the votes of every
//                    distinct token and ranks (votes desc, index asc) by comparison in LDS;
//   vote_count / vote_composite / vote_pick
//                    more votes (a chunk of query rows): atomic counts in a dense array over
//                    the middle, the thread that finds a zero lists the token, then one
//                    workgroup radix-selects the k' largest (votes, ~index) composites;
//   centres_to_spans (tail of both) sorted centres -> clipped spans -> union by prefix maximum
//                    / prefix sum -> ascending index list and its length (a device scalar: the
//                    scope of the following attention is data dependent).
#include "common.hpp"
#include "select.hpp"
#include "vote_scan.hpp"

namespace reattn {
namespace {


// ---- the same scan on the matrix cores (bf16, D = 128) ----------------------------------
// A key tile of 16 rows is the A operand of v_mfma_f32_16x16x32_bf16 and up to 16 (query row,
// head) pairs of one KV head are the columns of B, so one MFMA chain of 4 gives 16 x 16 raw
// scores and the vector ALU only compares: the stream stays HBM-bound however many heads vote.
// For step j of the chain lane l supplies the 16-byte piece 4j + l/16 of key row l%16 (the
// contraction does not care which 8 channels sit in which k slot as long as B uses the same
// assignment).  Loading the keys from memory in that shape (16 rows x 64 bytes per
// instruction) tops out at 6.0 TB/s; 1 KiB of consecutive memory per instruction reaches
// 6.9, so tiles are loaded that way and turned into the operand shape through a wave-private,
// XOR-swizzled LDS stage (no barrier: a wave reads only what it wrote).  The product leaves
// lane l with the scores of column l%16 against key rows 4(l/16)..+3: one running list per
// lane and column block, merged over the four lanes of a column, then over the waves.
typedef __bf16 bf16x8 __attribute__((ext_vector_type(8)));
typedef float f32x4 __attribute__((ext_vector_type(4)));

constexpr int kMfmaTiles = 2;                          // key tiles (16 rows) per wave iteration

struct MfmaScanArgs {
  const void* k; const void* q;
  uint64_t* part;          // [n_query * Hq][n_wg][KT] composites, best first
  int64_t ksh, kst, n_mid, first_tok;
  int Hq, Hkv, G, n_query, q_per_pass, rows_per_block, n_wg;
  const int32_t* pt; int page_lg;   // paged cache (PAGED kernels)
};

template <int KT, int NB, bool F16, bool PAGED = false>
__global__ __launch_bounds__(kVoteThreads) void head_topk_mfma_kernel(MfmaScanArgs a) {
  typedef typename Mm<F16>::op8 op8;
  __shared__ int32_t s_pages[PAGED ? kVotePages : 1];
  constexpr int D = 128, T = kMfmaTiles, NC = 16 * NB;
  // staging of the key tiles [kVoteWaves][T][16 rows][16 pieces] of 16 bytes while streaming,
  // then the waves' merged lists [kVoteWaves][NC][KT]
  extern __shared__ __attribute__((aligned(16))) uint64_t mfma_lds[];
  uint64_t* mfma_best = mfma_lds;
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  const int col = lane & 15, kq = lane >> 4;
  const int h = blockIdx.y % a.Hkv, q0 = (blockIdx.y / a.Hkv) * a.q_per_pass;
  const int q_here = a.n_query - q0 < a.q_per_pass ? a.n_query - q0 : a.q_per_pass;
  const int n_cols = q_here * a.G;

  op8 bq[NB][4];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
    const int c = nb * 16 + col;
    const bool live = c < n_cols;
    const int64_t row = live ? ((int64_t)(q0 + c / a.G) * a.Hq + (int64_t)h * a.G + c % a.G) : 0;
    const u32x4* src = (const u32x4*)((const uint16_t*)a.q + row * D);
#pragma unroll
    for (int j = 0; j < 4; ++j) {
      u32x4 w = src[4 * j + kq];
      if (!live) w = u32x4{0u, 0u, 0u, 0u};
      bq[nb][j] = __builtin_bit_cast(op8, w);
    }
  }
  float bv[NB][KT]; uint32_t bi[NB][KT];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb)
#pragma unroll
    for (int t = 0; t < KT; ++t) { bv[nb][t] = -__builtin_inff(); bi[nb][t] = 0xffffffffu; }

  const int64_t blk_row0 = (int64_t)blockIdx.x * a.rows_per_block;
  const int64_t left = a.n_mid - blk_row0;
  const int nrows = left < a.rows_per_block ? (int)left : a.rows_per_block;
  const int64_t row_bytes = a.kst * 2;
  const int64_t tok0 = a.first_tok + blk_row0;
  const char* kbase = (const char*)a.k + ((int64_t)h * a.ksh + (PAGED ? 0 : tok0) * a.kst) * 2 + col * 16;
  if (PAGED) slice_pages_fill(s_pages, a.pt, a.page_lg, tok0, nrows, kVoteThreads);
  static_assert(16 * T <= 64, "a wave's tile lies in at most two pages");
  u32x4* my = (u32x4*)mfma_lds + wave * (T * 256);     // this wave's T tiles of 16 rows x 16 pieces

  // global -> registers: 1 KiB of consecutive memory per load (lane l: row l/16, piece l%16); the loads
  // of the next iteration are in flight while this one is contracted and sifted
  auto request = [&](int t, u32x4* d) {
    TilePages tp;
    if (PAGED) tp = tile_pages(s_pages, a.page_lg, tok0, tok0 + t);
#pragma unroll
    for (int u = 0; u < 4 * T; ++u) {
      int r = t + u * 4 + kq;
      r = r < nrows ? r : nrows - 1;                   // tail rows re-read the last row; result dropped
      const int64_t row = PAGED ? tp.row(r - t) : r;
      d[u] = __builtin_nontemporal_load((const u32x4*)(kbase + row * row_bytes));
    }
  };
  constexpr bool kAhead = NB == 1;                     // two column blocks leave no registers for a second batch
  u32x4 d[4 * T], dn[kAhead ? 4 * T : 1];
  if (kAhead && wave * (T * 16) < nrows) request(wave * (T * 16), d);
  for (int t = wave * (T * 16); t < nrows; t += kVoteWaves * (T * 16)) {
    if (kAhead) {
      const int t_next = t + kVoteWaves * (T * 16);
      if (t_next < nrows) request(t_next, dn);
    } else {
      request(t, d);
    }
    // registers -> wave-private LDS, piece index XOR row so that both sides are conflict free
#pragma unroll
    for (int u = 0; u < 4 * T; ++u) {
      const int row = u * 4 + kq;
      my[row * 16 + (col ^ (row & 15))] = d[u];
    }
#pragma unroll
    for (int tt = 0; tt < T; ++tt) {
      const int r0 = t + tt * 16 + kq * 4;             // this lane's four key rows of the tile
      u32x4 ka[4];                                     // LDS -> A operand: row l%16, piece 4j + l/16
#pragma unroll
      for (int j = 0; j < 4; ++j) ka[j] = my[(tt * 16 + col) * 16 + ((4 * j + kq) ^ col)];
#pragma unroll
      for (int nb = 0; nb < NB; ++nb) {
        f32x4 acc = {0.f, 0.f, 0.f, 0.f};
#pragma unroll
        for (int j = 0; j < 4; ++j)
          acc = Mm<F16>::mfma16(__builtin_bit_cast(op8, ka[j]), bq[nb][j], acc);
        const float m01 = acc[0] > acc[1] ? acc[0] : acc[1], m23 = acc[2] > acc[3] ? acc[2] : acc[3];
        if ((m01 > m23 ? m01 : m23) > bv[nb][KT - 1]) {
#pragma unroll
          for (int i = 0; i < 4; ++i) {
            // rows arrive in ascending position per lane: a later equal score never displaces
            if (r0 + i < nrows && acc[i] > bv[nb][KT - 1]) {
              bv[nb][KT - 1] = acc[i]; bi[nb][KT - 1] = (uint32_t)(blk_row0 + r0 + i);
#pragma unroll
              for (int x = KT - 1; x > 0; --x) {
                if (bv[nb][x] > bv[nb][x - 1]) {
                  const float fv = bv[nb][x]; bv[nb][x] = bv[nb][x - 1]; bv[nb][x - 1] = fv;
                  const uint32_t iv = bi[nb][x]; bi[nb][x] = bi[nb][x - 1]; bi[nb][x - 1] = iv;
                }
              }
            }
          }
        }
      }
    }
    if (kAhead) {
#pragma unroll
      for (int u = 0; u < 4 * T; ++u) d[u] = dn[kAhead ? u : 0];
    }
  }

  // the four lanes of a column merge their lists: KT rounds of arg-max over lanes l, l^16, l^32, l^48
  uint64_t keep[NB][KT];
#pragma unroll
  for (int nb = 0; nb < NB; ++nb) {
#pragma unroll
    for (int round = 0; round < KT; ++round) {
      const uint64_t c = bi[nb][0] != 0xffffffffu ? composite(bv[nb][0], bi[nb][0]) : 0ull;
      uint64_t best = c;
#pragma unroll
      for (int o = 16; o <= 32; o <<= 1) {
        const uint32_t lo = __shfl_xor((uint32_t)best, o, 64), hi = __shfl_xor((uint32_t)(best >> 32), o, 64);
        const uint64_t w = ((uint64_t)hi << 32) | lo;
        best = w > best ? w : best;
      }
      if (c == best && best != 0ull) {                 // pop: composites are unique (distinct positions)
#pragma unroll
        for (int x = 0; x + 1 < KT; ++x) { bv[nb][x] = bv[nb][x + 1]; bi[nb][x] = bi[nb][x + 1]; }
        bv[nb][KT - 1] = -__builtin_inff(); bi[nb][KT - 1] = 0xffffffffu;
      }
      keep[nb][round] = best;
    }
  }
  __syncthreads();                                     // every wave is done with its staging area
  if (kq == 0) {
#pragma unroll
    for (int nb = 0; nb < NB; ++nb)
#pragma unroll
      for (int round = 0; round < KT; ++round)
        mfma_best[((size_t)wave * NC + nb * 16 + col) * KT + round] = keep[nb][round];
  }
  __syncthreads();
  // workgroup merge: a wave takes every 16th column; its lanes hold the 16 waves' KT entries
  for (int c = wave; c < n_cols; c += kVoteWaves) {
    uint64_t c0 = 0ull, c1 = 0ull;
    if (lane < kVoteWaves * KT) c0 = mfma_best[((size_t)(lane / KT) * NC + c) * KT + lane % KT];
    if (lane + 64 < kVoteWaves * KT) c1 = mfma_best[((size_t)((lane + 64) / KT) * NC + c) * KT + (lane + 64) % KT];
    uint64_t* out = a.part +
        (((int64_t)(q0 + c / a.G) * a.Hq + (int64_t)h * a.G + c % a.G) * a.n_wg + blockIdx.x) * KT;
#pragma unroll
    for (int round = 0; round < KT; ++round) {
      const uint64_t best = wave_max_u64(c0 > c1 ? c0 : c1);
      if (c0 == best) c0 = 0ull;
      if (c1 == best) c1 = 0ull;
      if (lane == 0) out[round] = best;
    }
  }
}

// One wave per (query, head): best vote_k of n_wg * KT composites -> ascending absolute indices.
__global__ __launch_bounds__(64) void head_topk_merge_kernel(const uint64_t* __restrict__ part, int n_cand,
                                                             int vote_k, int32_t index_base,
                                                             int32_t* head_topk) {
  const int lane = threadIdx.x;
  const uint64_t* p = part + (int64_t)blockIdx.x * n_cand;
  uint32_t mine = 0xffffffffu;                         // lane t < vote_k ends up with the t-th best position
  uint64_t taken_below = ~0ull;                        // composites are distinct: walk down strictly
  for (int round = 0; round < vote_k; ++round) {
    uint64_t c = 0ull;
    for (int i = lane; i < n_cand; i += 64) {
      const uint64_t v = p[i];
      if (v < taken_below && v > c) c = v;
    }
    const uint64_t best = wave_max_u64(c);
    taken_below = best;
    if (lane == round) mine = best ? 0xffffffffu - (uint32_t)best : 0xffffffffu;
  }
  // ascending order: rank of each kept position among the kept ones
  int rank = 0;
  for (int t = 0; t < vote_k; ++t) {
    const uint32_t o = __shfl(mine, t, 64);
    rank += (o < mine) ? 1 : 0;
  }
  if (lane < vote_k) head_topk[(int64_t)blockIdx.x * vote_k + rank] = index_base + (int32_t)mine;
}

// ---- votes -> centres -> spans ---------------------------------------------------------
// Composite of a voted token: (votes desc, index asc) as one unsigned maximum; 0 = nothing.
__device__ __forceinline__ uint64_t vote_composite(uint32_t votes, uint32_t tok) {
  return ((uint64_t)votes << 32) | (uint64_t)(0xffffffffu - tok);
}

constexpr int kMergeThreads = 1024;     // also the largest number of centres
constexpr int kPickCache = 12288;       // composites the dense pick keeps in LDS (96 KiB)
constexpr size_t kPickLds = (size_t)kPickCache * 8 + 2048 * 4;

struct SpanArgs {
  int32_t s_eff; int64_t n_mid; int kc, span;
  int32_t* sel; int32_t* n_sel;
};

template <bool MAX, int NT>
__device__ __forceinline__ int32_t block_scan_i32(int32_t v, int32_t* wsum) {   // inclusive, NT threads
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  int32_t x = v;
#pragma unroll
  for (int o = 1; o < 64; o <<= 1) {
    const int32_t y = __shfl_up(x, o, 64);
    if (lane >= o) x = MAX ? (x > y ? x : y) : x + y;
  }
  if (lane == 63) wsum[wave] = x;
  __syncthreads();
  int32_t base = 0;
#pragma unroll
  for (int w = 0; w < NT / 64; ++w) {
    const int32_t s = wsum[w];
    if (w < wave) base = MAX ? (base > s ? base : s) : base + s;
  }
  __syncthreads();
  return MAX ? (x > base ? x : base) : x + base;
}

// win[0 .. nc): the centres (distinct tokens relative to the middle, any order), nc <= NT.
// Sorts them, clips each span to the middle, unions overlapping spans (a span can only
// overlap spans of earlier centres once they ascend) and writes the ascending index list.
template <int NT>
__device__ __forceinline__ void centres_to_spans(int32_t* win, int nc, int32_t* sa, int32_t* sb,
                                                 int32_t* wsum, const SpanArgs& a) {
  const int i = threadIdx.x;
  const int32_t mine = i < nc ? win[i] : 0;
  int rank = 0;
  if (i < nc)                                          // the other waves skip the loop altogether
    for (int j = 0; j < nc; ++j) rank += win[j] < mine ? 1 : 0;
  __syncthreads();
  if (i < nc) sa[rank] = mine;                         // ascending centres
  __syncthreads();
  int32_t lo = 0, hi = 0;
  if (i < nc) {
    const int64_t l64 = (int64_t)sa[i] - a.span / 2, h64 = l64 + a.span;
    lo = (int32_t)(l64 < 0 ? 0 : l64);
    hi = (int32_t)(h64 > a.n_mid ? a.n_mid : h64);
  }
  __syncthreads();
  const int32_t hmax = block_scan_i32<true, NT>(hi, wsum);           // inclusive prefix maximum of hi
  sb[i] = hmax;
  __syncthreads();
  const int32_t before = i > 0 ? sb[i - 1] : 0;
  const int32_t start = lo > before ? lo : before;
  const int32_t len = hi > start ? hi - start : 0;
  __syncthreads();
  const int32_t end_at = block_scan_i32<false, NT>(len, wsum);       // inclusive prefix sum of lengths
  sa[i] = end_at; sb[i] = start - (end_at - len);                // output slot o of centre i holds sb[i] + o
  __syncthreads();
  const int32_t total = sa[NT - 1];
  for (int32_t o = i; o < total; o += NT) {
    int l = 0, h = NT - 1;                  // first centre whose inclusive end exceeds o
    while (l < h) {
      const int mid = (l + h) >> 1;
      if (sa[mid] > o) h = mid; else l = mid + 1;
    }
    a.sel[o] = a.s_eff + sb[l] + o;
  }
  if (i == 0) *a.n_sel = total;
}

// Up to NT votes and centres (a decode step: Hq * vote_k votes): everything in one workgroup, no vote array.
// v: this thread's vote as a token of the middle, or -1.
template <int NT>
__device__ __forceinline__ void small_merge(int32_t v, int n_votes, const SpanArgs& a, int32_t* tok, int32_t* win,
                                            int32_t* sa, int32_t* sb, uint64_t* comp, int32_t* wsum) {
  const int t = threadIdx.x;
  tok[t] = v;
  __syncthreads();
  uint32_t votes = 0;
  bool first = true;                                   // the earliest vote for a token stands for it
  if (v >= 0)                                          // waves without a vote skip the loops
    for (int j = 0; j < n_votes; ++j) {
      const int32_t x = tok[j];
      votes += x == v ? 1u : 0u;
      first = first && !(x == v && j < t);
    }
  const bool owner = v >= 0 && first;
  const uint64_t c = owner ? vote_composite(votes, (uint32_t)v) : 0ull;
  comp[t] = c;
  __syncthreads();
  int rank = 0;                                        // distinct tokens ahead of this one
  if (owner)
    for (int j = 0; j < n_votes; ++j) rank += comp[j] > c ? 1 : 0;
  const int n_owner = __syncthreads_count(owner);
  if (owner && rank < a.kc) win[rank] = v;             // composites are distinct: ranks are a permutation
  __syncthreads();
  centres_to_spans<NT>(win, n_owner < a.kc ? n_owner : a.kc, sa, sb, wsum, a);
}

// blockIdx.x is the sequence of a folded batch: its n_votes consecutive list entries, its own output row.
template <int NT>
__global__ __launch_bounds__(NT) void vote_merge_small_kernel(const int32_t* __restrict__ lists, int n_votes,
                                                              int64_t sel_stride, SpanArgs a) {
  lists += (int64_t)blockIdx.x * n_votes;
  a.sel += (int64_t)blockIdx.x * sel_stride;
  a.n_sel += blockIdx.x;
  __shared__ int32_t tok[NT], win[NT], sa[NT], sb[NT];
  __shared__ uint64_t comp[NT];
  __shared__ int32_t wsum[NT / 64];
  const int t = threadIdx.x;
  int32_t v = t < n_votes ? lists[t] - a.s_eff : -1;
  if (v < 0 || v >= a.n_mid) v = -1;                   // an entry outside the middle is no vote
  small_merge<NT>(v, n_votes, a, tok, win, sa, sb, comp, wsum);
}

// A decode step's selection after the scan, in one workgroup per sequence: every wave closes the lists of
// its heads (best vote_k of the n_cand composites the scan's workgroups left for the head), the votes are
// counted and the spans expanded as above, and the rows of the token being decoded are copied into the
// cache on the side (they are the last local entry: only the attention that follows reads them).
constexpr int kDecodeCand = 512;        // composites per head the one-workgroup decode merge holds in registers

// 1024 threads: sixteen waves close the lists side by side (a wave's reductions run one after another, and
// with four waves the eight heads each of them got made this the longest kernel of the step after the scan).
template <int NT>
__global__ __launch_bounds__(NT) void vote_decode_merge_kernel(const uint64_t* __restrict__ part, int n_cand,
                                                               int vote_k, int heads, int64_t sel_stride,
                                                               SpanArgs a, AppendArgs ap) {
  a.sel += (int64_t)blockIdx.x * sel_stride;
  a.n_sel += blockIdx.x;
  __shared__ int32_t tok[NT], win[NT], sa[NT], sb[NT];
  __shared__ uint64_t comp[NT];
  __shared__ int32_t wsum[NT / 64];
  const int t = threadIdx.x, lane = t & 63, wave = t >> 6;
  if (blockIdx.x == 0)
    for (int64_t i = t; i < ap.n_vec; i += NT) append_piece(ap, i);
  for (int h = wave; h < heads; h += NT / 64) {
    const uint64_t* p = part + ((int64_t)blockIdx.x * heads + h) * n_cand;
    uint64_t c[kDecodeCand / 64];                      // the head's composites, read once (clamped, then masked)
#pragma unroll
    for (int u = 0; u < kDecodeCand / 64; ++u) {
      const int i = u * 64 + lane;
      c[u] = p[i < n_cand ? i : n_cand - 1];
    }
#pragma unroll
    for (int u = 0; u < kDecodeCand / 64; ++u) c[u] = u * 64 + lane < n_cand ? c[u] : 0ull;
    uint64_t taken_below = ~0ull;                      // composites are distinct: walk down strictly
    uint32_t mine = 0xffffffffu;
    for (int round = 0; round < vote_k; ++round) {
      uint64_t m = 0ull;
#pragma unroll
      for (int u = 0; u < kDecodeCand / 64; ++u)
        if (c[u] < taken_below && c[u] > m) m = c[u];
      const uint64_t best = wave_max_u64(m);
      taken_below = best;
      if (lane == round) mine = best ? 0xffffffffu - (uint32_t)best : 0xffffffffu;
    }
    if (lane < vote_k) sa[h * vote_k + lane] = (mine != 0xffffffffu && (int64_t)mine < a.n_mid) ? (int32_t)mine : -1;
  }
  __syncthreads();
  const int n_votes = heads * vote_k;
  const int32_t v = t < n_votes ? sa[t] : -1;
  __syncthreads();                                     // sa is scratch of the span expansion from here on
  small_merge<NT>(v, n_votes, a, tok, win, sa, sb, comp, wsum);
}

// More votes than one workgroup ranks by comparison: a dense vote array over the middle.
// The thread whose atomic finds a zero stands for the token and lists it in its workgroup's
// segment; unused slots of the segment are marked.
__global__ __launch_bounds__(kMergeThreads) void vote_count_kernel(const int32_t* __restrict__ lists,
                                                                   int64_t n_votes, int32_t s_eff, int32_t n_mid,
                                                                   uint32_t* counts, int32_t* seg) {
  __shared__ uint32_t n_own;
  if (threadIdx.x == 0) n_own = 0;
  __syncthreads();
  const int64_t i = (int64_t)blockIdx.x * kMergeThreads + threadIdx.x;
  int32_t* my_seg = seg + (int64_t)blockIdx.x * kMergeThreads;
  if (i < n_votes) {
    const int32_t v = lists[i] - s_eff;
    if (v >= 0 && v < n_mid)                           // an entry outside the middle is no vote
      if (atomicAdd(&counts[v], 1u) == 0u) my_seg[atomicAdd(&n_own, 1u)] = v;
  }
  __syncthreads();
  if (threadIdx.x >= n_own) my_seg[threadIdx.x] = -1;
}

// Once every vote is counted: the composite of every listed token (0 in unused slots), and how
// many tokens hold each vote count (counts of kCountBins - 1 and more share the last bin).
constexpr int kCountBins = 2048;
__global__ __launch_bounds__(kMergeThreads) void vote_composite_kernel(const int32_t* __restrict__ seg,
                                                                       const uint32_t* __restrict__ counts,
                                                                       uint64_t* comp, uint32_t* chist) {
  __shared__ uint32_t lh[kCountBins];
  for (int b = threadIdx.x; b < kCountBins; b += kMergeThreads) lh[b] = 0;
  __syncthreads();
  const int64_t i = (int64_t)blockIdx.x * kMergeThreads + threadIdx.x;
  const int32_t v = seg[i];
  uint64_t c = 0ull;
  if (v >= 0) {
    const uint32_t n = counts[v];
    c = vote_composite(n, (uint32_t)v);
    atomicAdd(&lh[n < kCountBins - 1 ? n : kCountBins - 1], 1u);
  }
  comp[i] = c;
  __syncthreads();
  for (int b = threadIdx.x; b < kCountBins; b += kMergeThreads)
    if (lh[b]) atomicAdd(&chist[b], lh[b]);
}

// The histogram of vote counts names the count d of the kc-th token: everything above it wins
// outright, and the tokens holding exactly d are tied and decided by index.  Every workgroup
// finds d for itself (2048 bins) and sorts its 1024 composites into the winners' list and the
// list of tied tokens (one atomic per workgroup and list).  Nothing to do when the last bin,
// which mixes counts, holds the kc-th token: the pick then selects over all composites.
struct SiftOut {
  uint32_t* n_lists;     // [0] winners so far, [1] tied tokens so far (zeroed with the vote array)
  int32_t* winners;      // [kMergeThreads] tokens relative to the middle
  uint32_t* tied;        // low words (~index) of the tied tokens' composites
};

__device__ __forceinline__ void kth_count(const uint32_t* chist, int kc, uint32_t* sh, uint32_t& n, uint32_t& d,
                                          uint32_t& above) {
  const uint32_t x = chist[2 * threadIdx.x] + chist[2 * threadIdx.x + 1];
  block_scan_incl<kMergeThreads>(x, sh, n);
  d = 0; above = 0;
  if (n > (uint32_t)kc) find_kth_bin<kMergeThreads, kCountBins>(chist, (uint32_t)kc, sh, d, above);
}

__global__ __launch_bounds__(kMergeThreads) void vote_sift_kernel(const uint64_t* __restrict__ comp,
                                                                  const uint32_t* __restrict__ chist, int kc,
                                                                  SiftOut o) {
  __shared__ uint32_t sh[40];
  __shared__ uint32_t n_w, n_t, base_w, base_t;
  if (threadIdx.x == 0) { n_w = 0; n_t = 0; }
  uint32_t n, d, above;
  kth_count(chist, kc, sh, n, d, above);                        // includes barriers
  const bool all_win = n <= (uint32_t)kc;
  if (!all_win && d == kCountBins - 1) return;                  // saturated bins: left to the pick
  const uint64_t c = comp[(int64_t)blockIdx.x * kMergeThreads + threadIdx.x];
  const uint32_t votes = (uint32_t)(c >> 32);
  const bool wins = c != 0ull && (all_win || votes > d);
  const bool ties = c != 0ull && !all_win && votes == d;
  uint32_t my = 0;
  if (wins) my = atomicAdd(&n_w, 1u);
  if (ties) my = atomicAdd(&n_t, 1u);
  __syncthreads();
  if (threadIdx.x == 0) {
    base_w = n_w ? atomicAdd(&o.n_lists[0], n_w) : 0u;
    base_t = n_t ? atomicAdd(&o.n_lists[1], n_t) : 0u;
  }
  __syncthreads();
  if (wins) o.winners[base_w + my] = (int32_t)(0xffffffffu - (uint32_t)c);
  if (ties) o.tied[base_t + my] = (uint32_t)c;
}

// One workgroup: the winners, plus the lowest-indexed of the tied tokens (radix select on the
// composites' low words, the first kPickCache of them held in LDS), then sort + spans.  With
// saturated count bins: radix select over all composites (11-bit digits from `top_bit` down).
// n_slots is a multiple of 1024.
__global__ __launch_bounds__(kMergeThreads) void vote_pick_kernel(const uint64_t* __restrict__ comp,
                                                                  const uint32_t* __restrict__ chist, SiftOut o,
                                                                  int64_t n_slots, int top_bit, SpanArgs a) {
  extern __shared__ uint64_t pick_lds[];
  uint32_t* bins = (uint32_t*)(pick_lds + kPickCache);          // [2048]
  __shared__ int32_t win[kMergeThreads], sa[kMergeThreads], sb[kMergeThreads];
  __shared__ int32_t wsum[kMergeThreads / 64];
  __shared__ uint32_t sh[40];
  __shared__ uint32_t n_win;
  uint32_t n, d, above;
  kth_count(chist, a.kc, sh, n, d, above);
  const bool all_win = n <= (uint32_t)a.kc;
  if (all_win || d < kCountBins - 1) {
    uint32_t* cached = (uint32_t*)pick_lds;                     // [2 * kPickCache] low words
    constexpr uint32_t kCache = 2 * kPickCache;
    const uint32_t nw = o.n_lists[0], nt = all_win ? 0u : o.n_lists[1];
    if (threadIdx.x == 0) n_win = nw;
    if (threadIdx.x < nw) win[threadIdx.x] = o.winners[threadIdx.x];
    for (uint32_t i = threadIdx.x; i < nt && i < kCache; i += kMergeThreads) cached[i] = o.tied[i];
    __syncthreads();
    if (nt) {
      auto low = [&](uint32_t i) -> uint32_t { return i < kCache ? cached[i] : o.tied[i]; };
      const uint32_t need = (uint32_t)a.kc - above;             // lowest indices = largest low words
      int shift = 0;
      uint32_t prefix = 0;
      if (need < nt) {
        shift = 32;
        uint32_t remaining = need;
        while (shift > 0) {
          const int w = shift < 11 ? shift : 11;
          shift -= w;
          for (int b = threadIdx.x; b < 2048; b += kMergeThreads) bins[b] = 0;
          __syncthreads();
          for (uint32_t i = threadIdx.x; i < nt; i += kMergeThreads) {
            const uint64_t c = low(i);
            if ((uint32_t)(c >> (shift + w)) == prefix) atomicAdd(&bins[(uint32_t)(c >> shift) & ((1u << w) - 1u)], 1u);
          }
          __syncthreads();
          uint32_t dd, ab;
          find_kth_bin<kMergeThreads, 2048>(bins, remaining, sh, dd, ab);
          const uint32_t in_bin = bins[dd];
          remaining -= ab;
          prefix = (prefix << w) | dd;
          __syncthreads();
          if (in_bin == remaining) break;
        }
      }
      for (uint32_t i = threadIdx.x; i < nt; i += kMergeThreads) {
        const uint32_t c = low(i);
        if ((shift >= 32 ? 0u : c >> shift) >= prefix) win[atomicAdd(&n_win, 1u)] = (int32_t)(0xffffffffu - c);
      }
    }
    __syncthreads();
    centres_to_spans<kMergeThreads>(win, (int)n_win, sa, sb, wsum, a);
    return;
  }

  // ---- saturated count bins: radix select over all composites ----
  uint64_t* cached = pick_lds;                                  // [kPickCache]
  if (threadIdx.x == 0) n_win = 0;
  for (int64_t i = threadIdx.x; i < n_slots && i < kPickCache; i += kMergeThreads) cached[i] = comp[i];
  __syncthreads();
  auto at = [&](int64_t i) -> uint64_t { return i < kPickCache ? cached[i] : comp[i]; };
  int shift = top_bit;
  uint64_t prefix = 0;                                          // winners: c != 0 and (c >> shift) >= prefix
  uint32_t remaining = (uint32_t)a.kc;
  while (shift > 0) {
    const int w = shift < 11 ? shift : 11;
    shift -= w;
    for (int b = threadIdx.x; b < 2048; b += kMergeThreads) bins[b] = 0;
    __syncthreads();
    for (int64_t i = threadIdx.x; i < n_slots; i += kMergeThreads) {
      const uint64_t c = at(i);
      if (c && (c >> (shift + w)) == prefix)
        atomicAdd(&bins[(uint32_t)(c >> shift) & ((1u << w) - 1u)], 1u);
    }
    __syncthreads();
    uint32_t dd, ab;
    find_kth_bin<kMergeThreads, 2048>(bins, remaining, sh, dd, ab);
    const uint32_t in_bin = bins[dd];
    remaining -= ab;
    prefix = (prefix << w) | dd;
    __syncthreads();
    if (in_bin == remaining) break;                             // everything sharing this prefix wins
  }
  for (int64_t i = threadIdx.x; i < n_slots; i += kMergeThreads) {
    const uint64_t c = at(i);
    if (c && (c >> shift) >= prefix) win[atomicAdd(&n_win, 1u)] = (int32_t)(0xffffffffu - (uint32_t)c);
  }
  __syncthreads();
  centres_to_spans<kMergeThreads>(win, (int)n_win, sa, sb, wsum, a);
}

}  // namespace

int scan_rows_per_block(int64_t n_mid, int64_t score_rows, int max_rows);

int vote_list_len(int vote_k) { return vote_k <= 1 ? 1 : vote_k <= 2 ? 2 : vote_k <= 4 ? 4 : 8; }

// Every shape the library takes: 16-bit storage with D = 128 on the matrix cores, the rest on the vector ALU.
bool vote_scan_applies(const Plan& pl) { return pl.G <= 16; }

// Geometry of one scan launch over n_query query rows.
struct ScanGeom { bool mfma, gemm; int nb, q_per_pass, n_pass, rpb, n_wg; };

ScanGeom scan_geom(const Plan& pl, int n_query, int kt) {
  ScanGeom g;
  g.mfma = pl.dtype != kF32 && pl.D == 128;
  g.gemm = g.mfma && n_query * pl.G > 32;              // more columns than one streaming pass holds
  if (g.gemm) {                                        // tiled contraction: every key is read once per workgroup of 256 or 512 columns
    g.nb = 0; g.q_per_pass = n_query; g.n_pass = 1; g.rpb = 0;
    g.n_wg = vote_gemm_splits(pl, n_query, kt);
    return g;
  }
  if (g.mfma) {
    g.nb = n_query * pl.G <= 16 ? 1 : 2;               // column blocks of 16 (query row, head) pairs
    g.q_per_pass = 16 * g.nb / pl.G;
    g.n_pass = (n_query + g.q_per_pass - 1) / g.q_per_pass;
  } else {
    g.nb = 0; g.q_per_pass = 1; g.n_pass = n_query;    // the vector-ALU scan streams once per query row
  }
  // nothing is parked in LDS here: slices of 16K rows (two rounds at 1M tokens) stream a little faster
  g.rpb = scan_rows_per_block(pl.n_mid, (int64_t)pl.Hkv * g.n_pass, 16384);
  g.n_wg = (int)((pl.n_mid + g.rpb - 1) / g.rpb);
  return g;
}

// Query rows one launch may take: grid.y = passes * Hkv stays below 65536.
int vote_queries_per_launch(const Plan& pl, int vote_k) {
  const ScanGeom one = scan_geom(pl, pl.M, vote_list_len(vote_k));
  if (one.gemm) return pl.M;
  const int64_t per = (int64_t)(65535 / pl.Hkv) * one.q_per_pass;
  return (int)(per < pl.M ? per : pl.M);
}

size_t vote_part_bytes(const Plan& pl, int n_query, int vote_k) {
  return (size_t)n_query * pl.Hq * scan_geom(pl, n_query, vote_list_len(vote_k)).n_wg * vote_list_len(vote_k) * sizeof(uint64_t);
}

template <int KT, bool F16>
hipError_t mfma_launch_nb(const MfmaScanArgs& a, int nb, dim3 grid, hipStream_t st) {
  const size_t lds = (size_t)kVoteWaves * kMfmaTiles * 256 * 16;      // staging; the merged lists fit inside
  static_assert((size_t)kVoteWaves * 32 * 8 * sizeof(uint64_t) <= (size_t)kVoteWaves * kMfmaTiles * 256 * 16, "lists alias the staging");
  auto k1 = head_topk_mfma_kernel<KT, 1, F16>;
  auto k2 = head_topk_mfma_kernel<KT, 2, F16>;
  auto p1 = head_topk_mfma_kernel<KT, 1, F16, true>;      // the same over a paged cache
  auto p2 = head_topk_mfma_kernel<KT, 2, F16, true>;
  const void* kern = a.pt ? (nb == 1 ? (const void*)p1 : (const void*)p2) : (nb == 1 ? (const void*)k1 : (const void*)k2);
  hipError_t e = hipFuncSetAttribute(kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  if (a.pt) {
    if (nb == 1) hipLaunchKernelGGL(p1, grid, dim3(kVoteThreads), lds, st, a);
    else         hipLaunchKernelGGL(p2, grid, dim3(kVoteThreads), lds, st, a);
  } else {
    if (nb == 1) hipLaunchKernelGGL(k1, grid, dim3(kVoteThreads), lds, st, a);
    else         hipLaunchKernelGGL(k2, grid, dim3(kVoteThreads), lds, st, a);
  }
  return hipGetLastError();
}
template <bool F16>
hipError_t mfma_launch_kt(const MfmaScanArgs& a, int kt, int nb, dim3 grid, hipStream_t st) {
  return kt == 1 ? mfma_launch_nb<1, F16>(a, nb, grid, st) : kt == 2 ? mfma_launch_nb<2, F16>(a, nb, grid, st)
       : kt == 4 ? mfma_launch_nb<4, F16>(a, nb, grid, st) : mfma_launch_nb<8, F16>(a, nb, grid, st);
}

// head_topk[i][hq][vote_k] for queries [0, n_query): ascending absolute indices.
namespace {
// The scan alone: every workgroup leaves its partial lists in `part`; *n_cand = composites per (query, head).
hipError_t launch_head_scan(const Plan& pl, const void* q, int n_query, const void* k_cache, int vote_k,
                            uint64_t* part, int* n_cand, hipStream_t st) {
  const int kt = vote_list_len(vote_k);
  const ScanGeom g = scan_geom(pl, n_query, kt);
  const dim3 grid((unsigned)(g.n_wg > 0 ? g.n_wg : 1), (unsigned)(pl.Hkv * g.n_pass));
  hipError_t e;
  if (g.gemm) {
    e = launch_vote_gemm(pl, q, n_query, k_cache, kt, part, st);
  } else if (g.mfma) {
    MfmaScanArgs a;
    a.k = k_cache; a.q = q; a.part = part;
    a.ksh = pl.ksh; a.kst = pl.kst; a.n_mid = pl.n_mid; a.first_tok = pl.s_eff;
    a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.G = pl.G; a.n_query = n_query; a.q_per_pass = g.q_per_pass;
    a.rows_per_block = g.rpb; a.n_wg = g.n_wg; a.pt = pl.pt; a.page_lg = pl.page_lg;
    e = pl.dtype == kF16 ? mfma_launch_kt<true>(a, kt, g.nb, grid, st) : mfma_launch_kt<false>(a, kt, g.nb, grid, st);
  } else {
    HeadScanArgs a;
    a.k = k_cache; a.q = q; a.part = part;
    a.ksh = pl.ksh; a.kst = pl.kst; a.n_mid = pl.n_mid; a.first_tok = pl.s_eff;
    a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.G = pl.G;
    a.rows_per_block = g.rpb; a.n_wg = g.n_wg; a.pt = pl.pt; a.page_lg = pl.page_lg;
    e = launch_head_scan_valu(pl, a, kt, grid, st);
  }
  *n_cand = g.n_wg * kt;
  return e;
}
}  // namespace

hipError_t launch_head_topk_scan(const Plan& pl, const void* q, int n_query, const void* k_cache,
                                 int vote_k, uint64_t* part, int32_t* head_topk, hipStream_t st) {
  if (pl.n_mid <= 0 || n_query <= 0 || vote_k <= 0) return hipSuccess;
  int n_cand = 0;
  hipError_t e = launch_head_scan(pl, q, n_query, k_cache, vote_k, part, &n_cand, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(head_topk_merge_kernel, dim3((unsigned)(n_query * pl.Hq)), dim3(64), 0, st, part,
                     n_cand, vote_k, (int32_t)pl.s_eff, head_topk);
  return hipGetLastError();
}

bool vote_decode_applies(const Plan& pl, int kk, int kc, int n_seq) {
  if (n_seq < 1) n_seq = 1;
  if (!(pl.M == 1 && pl.n_mid > 0 && kk > 0 && kc > 0 && kc <= kMergeThreads && pl.Hq % n_seq == 0 &&
        (int64_t)(pl.Hq / n_seq) * kk <= kMergeThreads))
    return false;
  const int kt = vote_list_len(kk);
  return scan_geom(pl, 1, kt).n_wg * kt <= kDecodeCand;
}

hipError_t launch_vote_decode_scan(const Plan& pl, const void* q, const void* k_cache, int kk, uint64_t* part,
                                   int* n_cand, hipStream_t st) {
  return launch_head_scan(pl, q, 1, k_cache, kk, part, n_cand, st);
}

hipError_t launch_vote_decode_merge(const Plan& pl, const uint64_t* part, int n_cand, int kk, int kc, int span,
                                    int32_t* sel, int32_t* n_sel, hipStream_t st, int n_seq, int64_t sel_stride,
                                    const AppendJob* append) {
  if (n_seq < 1) n_seq = 1;
  SpanArgs a;
  a.s_eff = (int32_t)pl.s_eff; a.n_mid = pl.n_mid; a.kc = kc; a.span = span; a.sel = sel; a.n_sel = n_sel;
  hipLaunchKernelGGL(vote_decode_merge_kernel<kMergeThreads>, dim3((unsigned)n_seq), dim3(kMergeThreads), 0, st, part,
                     n_cand, kk, pl.Hq / n_seq, sel_stride, a, append_args(pl, append));
  return hipGetLastError();
}

// Bytes of the dense vote array, the owner segments and their composites (0 for the small path).
void vote_merge_layout(const Plan& pl, int64_t n_votes, size_t* counts_bytes, size_t* seg_bytes,
                       size_t* comp_bytes) {
  const bool dense = n_votes > kMergeThreads && pl.n_mid > 0;
  const size_t slots = dense ? (size_t)((n_votes + kMergeThreads - 1) / kMergeThreads) * kMergeThreads : 0;
  // the vote array, the histogram of counts, two list lengths, the winners' list
  *counts_bytes = dense ? ((size_t)pl.n_mid + kCountBins + 2 + kMergeThreads) * 4 : 0;
  *seg_bytes = slots * 4;
  *comp_bytes = slots * 8;
}

// lists: n_rows lists of kk absolute indices.  kc centres (<= 1024), span m.
hipError_t launch_vote_merge(const Plan& pl, const int32_t* lists, int64_t n_rows, int kk, int kc, int span,
                             uint32_t* counts, int32_t* seg, uint64_t* comp, int32_t* sel, int32_t* n_sel,
                             hipStream_t st, int n_seq, int64_t sel_stride) {
  if (n_seq > 1) n_rows /= n_seq;                      // per sequence; only the one-workgroup path is batched
  const int64_t n_votes = n_rows * kk;
  if (n_seq > 1 && n_votes > kMergeThreads) return hipErrorInvalidValue;
  SpanArgs a;
  a.s_eff = (int32_t)pl.s_eff; a.n_mid = pl.n_mid; a.kc = kc; a.span = span; a.sel = sel; a.n_sel = n_sel;
  if (n_votes <= kMergeThreads) {
    if (n_votes <= 256 && kc <= 256)                   // a decode step: fewer waves, cheaper barriers
      hipLaunchKernelGGL(vote_merge_small_kernel<256>, dim3((unsigned)n_seq), dim3(256), 0, st, lists, (int)n_votes,
                         sel_stride, a);
    else
      hipLaunchKernelGGL(vote_merge_small_kernel<kMergeThreads>, dim3((unsigned)n_seq), dim3(kMergeThreads), 0, st,
                         lists, (int)n_votes, sel_stride, a);
    return hipGetLastError();
  }
  {
    hipError_t e = hipFuncSetAttribute((const void*)vote_pick_kernel,
                                       hipFuncAttributeMaxDynamicSharedMemorySize, (int)kPickLds);
    if (e != hipSuccess) return e;
  }
  const unsigned n_blocks = (unsigned)((n_votes + kMergeThreads - 1) / kMergeThreads);
  uint32_t* chist = counts + pl.n_mid;
  SiftOut so;
  so.n_lists = chist + kCountBins; so.winners = (int32_t*)(so.n_lists + 2);
  so.tied = (uint32_t*)seg;                            // the segments are spent once the composites exist
  hipError_t e = launch_fill_u32(counts, pl.n_mid + kCountBins + 2, 0u, st);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(vote_count_kernel, dim3(n_blocks), dim3(kMergeThreads), 0, st, lists, n_votes,
                     (int32_t)pl.s_eff, (int32_t)pl.n_mid, counts, seg);
  hipLaunchKernelGGL(vote_composite_kernel, dim3(n_blocks), dim3(kMergeThreads), 0, st, seg, counts, comp, chist);
  int top_bit = 33;                                    // 32 index bits + the bits of the largest vote count
  while (top_bit < 63 && (n_rows >> (top_bit - 32)) != 0) ++top_bit;
  hipLaunchKernelGGL(vote_sift_kernel, dim3(n_blocks), dim3(kMergeThreads), 0, st, comp, chist, kc, so);
  hipLaunchKernelGGL(vote_pick_kernel, dim3(1), dim3(kMergeThreads), kPickLds, st, comp, chist, so,
                     (int64_t)n_blocks * kMergeThreads, top_bit, a);
  return hipGetLastError();
}

}  // namespace reattn
