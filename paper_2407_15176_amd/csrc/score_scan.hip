// Stage 1 for a decode step: position-agnostic scores of one query against the
// whole middle of the key cache (paper Eq. 2, first line; appendix decoding
// phase, the `score = query @ key[l_global:-l_local]^T` line), summed over the
// heads of each GQA group.
//
// The kernel is a pure HBM stream: every key row (D elements, 128..512 bytes) is
// read exactly once with 16-byte non-temporal loads, LANES_PER_ROW adjacent lanes
// cover one row so each wave-wide load instruction fetches 1 KiB of consecutive
// memory, and the partial dot products are reduced with DPP row operations (no
// LDS round trip).  Because sum_g (q_g . k) = (sum_g q_g) . k, the group's query
// rows are summed once in fp32 registers and each key costs one dot product.
//
// Launch shape: one 1024-thread workgroup per CU, each owning one contiguous
// slice of one KV head.  Its scores (4 bytes per 256-byte row) are parked in LDS
// (up to 128 KiB) while it streams and are written out in one burst at the end:
// on MI355X any store issued in the middle of the stream costs ~15 % of the read
// bandwidth (dirty-line write-backs interleave with the reads), whereas a burst
// after the stream is nearly free.  The first radix digit of the top-k (a
// 4096-bin histogram of the ordered score keys) is accumulated in LDS on the way
// and flushed with one atomic per non-empty bin.
// Filter mode (no score array: only the pairs at or above a sampled bound leave the kernel) has nothing to
// write during the stream and runs two 512-thread workgroups per CU instead: one of the pair looks for its
// row's bound before it streams, the other behind its stream, so the CU's loads never stop for both
// (measured: 1.3 us of 326 per launch at a million tokens; all workgroups searching first: nothing).
#include "common.hpp"
#include "select.hpp"

namespace reattn {
namespace {

struct ScanArgs {
  const void* k;
  const void* q;
  float* scores;
  uint32_t* hist;       // [rows][kHistBins] or nullptr
  int64_t ksh, kst;     // key strides in elements
  int64_t n_mid, first_tok;
  int Hq, Hkv, G;
  int agg_max;          // REATTN_AGG_MAX: largest per-head dot product instead of their sum (MAXAGG kernels only)
  int rows_per_block;
  int stream_out;       // scores leave with non-temporal stores (several rounds of workgroups: a round's burst
                        // falls into the next round's reads, and ordinary stores would cost those ~9 %)
  const int32_t* pt;    // paged cache: the page of every 2^page_lg tokens of the sequence (PAGED kernels only)
  int page_lg;
  AppendArgs ap;        // rows of new tokens (past the middle) to copy into the caches on the way; n_vec 0: none
  // filter mode: instead of the scores, every slice leaves the (score, middle position) pairs at or above a
  // lower bound of the row's k-th score, in position order, in its own segment of rows_per_block entries
  const float* samp;    // [rows][samp_stride] scores of a strided sample of the row's keys
  int64_t samp_stride;
  uint32_t n_samp, rho; // the bound is (at most a hair below) the rho-th largest of the n_samp sampled scores
  uint2* cand;          // [rows][gridDim.x][rows_per_block]
  uint32_t* segcnt;     // [rows][gridDim.x]
};

constexpr int kScanThreads = 1024;
constexpr int kScanMaxRows = 32768;            // rows of scores one workgroup parks in LDS (128 KiB)

// How a slice's scores leave the workgroup.
constexpr int kOutScores = 0;                  // written as they are
constexpr int kOutHist = 1;                    // written, and the first radix digit of the top-k counted on the way
constexpr int kOutFilter = 2;                  // not written: only the pairs that can still be among the k largest
constexpr int kFilterThreads = 512;            // filter mode: two workgroups per CU, so that one streams while the other looks for its bound or compacts

// PAGED: the rows of a workgroup's slice are found through the page table; the few entries the slice
// spans are copied into LDS first, so a row costs one LDS read and two integer instructions more.
template <typename T, int D, int U, int MODE, bool PAGED = false, int NT = kScanThreads, bool MAXAGG = false>
__global__ __launch_bounds__(NT) void score_scan_kernel(ScanArgs a) {
  constexpr bool HIST = MODE == kOutHist, FILTER = MODE == kOutFilter;
  constexpr int kSampRegs = kFilterSampMax / NT;     // sampled scores a thread holds while the bound is found
  constexpr int EPL = Store<T>::kPerLoad;      // elements per 16-byte load
  constexpr int LPR = D / EPL;                 // lanes per key row
  constexpr int RPL = 64 / LPR;                // rows per wave-wide load
  constexpr int RW = U * RPL;                  // rows per wave iteration
  static_assert(U <= LPR, "one result slot per lane");

  extern __shared__ float stage[];             // [rows_per_block] scores (filter mode: one pad word per 32), then the histogram
  // filter mode: a thread later walks 32 consecutive scores; the pad word keeps those walks off each other's banks
  auto sidx = [](int r) -> int { return FILTER ? r + (r >> 5) : r; };
  uint32_t* lhist = (uint32_t*)(stage + (FILTER ? a.rows_per_block + (a.rows_per_block >> 5) + 1 : a.rows_per_block));
  uint32_t* fsh = lhist + kBinsPad;            // filter mode: lhist holds the select's 2048 padded bins, then 40 words
  if (a.ap.n_vec) {                            // a decode token's own rows: a few 16-byte pieces, copied first
    const int64_t n_thr = (int64_t)gridDim.x * gridDim.y * NT;
    for (int64_t i = ((int64_t)blockIdx.y * gridDim.x + blockIdx.x) * NT + threadIdx.x; i < a.ap.n_vec; i += n_thr)
      append_piece(a.ap, i);
  }
  if (HIST) {
    for (int b = threadIdx.x; b < kHistBins; b += NT) lhist[b] = 0;
    __syncthreads();
  }

  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int nwaves = NT / 64;
  const int sub = lane % LPR, grp = lane / LPR;
  const int row_id = blockIdx.y;               // query * Hkv + kv head
  const int h = row_id % a.Hkv, qi = row_id / a.Hkv;

  // The group's query rows, summed in fp32: this lane's EPL channels.
  float qv[EPL];
  if (!MAXAGG) group_query<T, D>(a.q, qi, h, a.Hq, a.G, sub, qv);

  // filter mode: the lower bound of the row's k-th score, from the sampled scores (every workgroup of the
  // row finds the same value; the sample is 36 KiB out of L2)
  // Two workgroups share a CU (the second round of workgroup ids lands beside the first): one looks for the
  // bound before its stream, the other behind it, so that the CU's loads never stop for both at once.
  uint32_t thr_key = 0;
  auto find_bound = [&]() {
    uint32_t skey[kSampRegs];
    const float* srow = a.samp + (int64_t)row_id * a.samp_stride;
#pragma unroll
    for (int r = 0; r < kSampRegs; ++r) {
      const uint32_t i = (uint32_t)r * NT + threadIdx.x;
      skey[r] = score_key(srow[i < a.n_samp ? i : a.n_samp - 1]);      // clamped, not predicated: the loads go out together
    }
    thr_key = kth_lower_bound_key<NT, kSampRegs>(skey, a.n_samp, a.rho, lhist, fsh);
  };
  const bool bound_first = (((blockIdx.y * gridDim.x + blockIdx.x) >> 8) & 1) == 0;
  if (FILTER && bound_first) find_bound();

  const int64_t blk_row0 = (int64_t)blockIdx.x * a.rows_per_block;
  const int64_t left = a.n_mid - blk_row0;
  const int nrows = left < a.rows_per_block ? (int)left : a.rows_per_block;
  const int64_t row_bytes = a.kst * (int64_t)sizeof(T);
  const char* kbase = (const char*)a.k +
      ((int64_t)h * a.ksh + (PAGED ? 0 : a.first_tok + blk_row0) * a.kst) * (int64_t)sizeof(T) + sub * 16;
  // paged: pages[i] = first row of page (pg0 + i) of the sequence, pg0 the page of the slice's first token
  int32_t* pages = (int32_t*)(lhist + (HIST ? kHistBins : FILTER ? kBinsPad + 40 : 0));
  const int64_t tok0 = a.first_tok + blk_row0;
  if (PAGED) slice_pages_fill(pages, a.pt, a.page_lg, tok0, nrows, NT);
  // max aggregation: the group's query rows, fp32, behind everything else in LDS
  float* qs = (float*)(pages + (PAGED ? (a.rows_per_block >> a.page_lg) + 3 : 0));
  float qr[MAXAGG ? 4 : 1][EPL];                        // ... or in registers when the group has at most four heads
  const bool few = a.G <= 4;
  if (MAXAGG) {
    if (few) {
      group_rows_to_regs<T, D>(a.q, qi, h, a.Hq, a.G, sub, qr);
    } else {
      group_rows_to_lds<T, D>(a.q, qi, h, a.Hq, a.G, qs, NT);
      __syncthreads();
    }
  }
  static_assert(RW <= 64, "a wave's tile lies in at most two pages");

  // heads start at different phases of their slices: the KV heads lie a power of two apart in a
  // contiguous cache, and workgroups of equal index would walk the same memory channels in step
  const int n_tile = (nrows + RW - 1) / RW;
  const int rot = (int)((int64_t)h * n_tile / a.Hkv);
  for (int it = wave; it < n_tile; it += nwaves) {
    const int tile = it + rot < n_tile ? it + rot : it + rot - n_tile;
    const int t = tile * RW;
    u32x4 d[U];
    TilePages tp;
    if (PAGED) tp = tile_pages(pages, a.page_lg, tok0, tok0 + t);
#pragma unroll
    for (int u = 0; u < U; ++u) {
      int r = t + u * RPL + grp;
      r = r < nrows ? r : nrows - 1;           // tail rows re-read the last row; result dropped
      const int64_t row = PAGED ? tp.row(r - t) : r;
      d[u] = __builtin_nontemporal_load((const u32x4*)(kbase + row * row_bytes));
    }
    float mine = 0.f;
#pragma unroll
    for (int u = 0; u < U; ++u) {
      float s;
      if (MAXAGG) {
        s = few ? row_dot_max4<T, D>(d[u], qr) : row_dot_max<T, D>(d[u], qs, a.G, sub);
      } else {
        float x[EPL];
        Store<T>::widen(d[u], x);
        s = 0.f;
#pragma unroll
        for (int e = 0; e < EPL; ++e) s = fmaf(x[e], qv[e], s);
        s = group_sum<LPR>(s);
      }
      mine = (sub == u) ? s : mine;            // lane (grp, sub) keeps the result of load `sub`
    }
    const int r = t + sub * RPL + grp;
    if (sub < U && r < nrows) {
      stage[sidx(r)] = mine;
      if (HIST) atomicAdd(&lhist[score_key(mine) >> kKeyShift], 1u);
    }
  }

  __syncthreads();
  if (FILTER) {
    if (!bound_first) find_bound();
    // ordered compaction out of LDS: thread t owns rows [32t, 32t + 32) of the slice
    const int r0 = (int)threadIdx.x * 32;
    uint32_t mask = 0;
#pragma unroll
    for (int i = 0; i < 32; ++i) {
      const int r = r0 + i < nrows ? r0 + i : (nrows > 0 ? nrows - 1 : 0);      // clamped: the LDS read stays inside the slice
      const bool in = r0 + i < nrows && score_key(stage[sidx(r)]) >= thr_key;
      mask |= in ? 1u << i : 0u;
    }
    const uint32_t mine = (uint32_t)__popc(mask);
    uint32_t total;
    uint32_t at = block_scan_incl<NT>(mine, fsh, total) - mine;
    const int64_t seg = (int64_t)row_id * gridDim.x + blockIdx.x;
    uint2* out = a.cand + seg * a.rows_per_block;
    while (mask) {
      const int i = __ffs((int)mask) - 1;
      mask &= mask - 1;
      out[at++] = make_uint2(__float_as_uint(stage[sidx(r0 + i)]), (uint32_t)(blk_row0 + r0 + i));
    }
    if (threadIdx.x == 0) a.segcnt[seg] = total;
    return;
  }
  float* out = a.scores + (int64_t)row_id * a.n_mid + blk_row0;
  if (a.stream_out) {
    for (int r = threadIdx.x; r < nrows; r += NT) __builtin_nontemporal_store(stage[r], out + r);
  } else {                                         // one round: the scores stay in cache for the top-k that follows
    for (int r = threadIdx.x; r < nrows; r += NT) out[r] = stage[r];
  }
  if (HIST) {
    uint32_t* gh = a.hist + (int64_t)row_id * kHistBins;
    for (int b = threadIdx.x; b < kHistBins; b += NT) {
      const uint32_t c = lhist[b];
      if (c) atomicAdd(&gh[b], c);
    }
  }
}

// Plain streaming read with the scan's load shape and nothing else: the ceiling the scan
// is normalised against in reports (no dot products, no stores).
__global__ __launch_bounds__(kScanThreads) void read_probe_kernel(const u32x4* __restrict__ p,
                                                                   size_t n_vec, size_t vec_per_block,
                                                                   uint32_t* sink) {
  const int lane = threadIdx.x & 63, wave = threadIdx.x >> 6;
  constexpr int U = 8, nwaves = kScanThreads / 64;
  size_t b0 = (size_t)blockIdx.x * vec_per_block, b1 = b0 + vec_per_block;
  if (b1 > n_vec) b1 = n_vec;
  uint32_t acc = 0;
  for (size_t t = b0 + (size_t)wave * U * 64; t < b1; t += (size_t)nwaves * U * 64) {
    u32x4 d[U];
#pragma unroll
    for (int u = 0; u < U; ++u) {
      size_t i = t + u * 64 + lane;
      if (i >= b1) i = b1 - 1;
      d[u] = __builtin_nontemporal_load(p + i);
    }
#pragma unroll
    for (int u = 0; u < U; ++u) acc += d[u].x ^ d[u].y ^ d[u].z ^ d[u].w;
  }
  if (acc == 0x9e3779b9u && sink) sink[0] = acc;   // keeps the loads alive; practically never taken
}

template <typename T, int D, int MODE, bool PAGED, bool MAXAGG>
hipError_t launch_hpa(const ScanArgs& a, dim3 grid, hipStream_t st) {
  constexpr int U = 8;
  const size_t lds = (size_t)a.rows_per_block * 4 + (MODE == kOutHist ? kHistBins * 4 : 0) +
                     (MODE == kOutFilter ? ((size_t)(a.rows_per_block >> 5) + 1 + kBinsPad + 40) * 4 : 0) +
                     (PAGED ? ((size_t)(a.rows_per_block >> a.page_lg) + 3) * 4 : 0) +
                     (MAXAGG ? (size_t)a.G * D * 4 : 0);
  constexpr int NT = MODE == kOutFilter ? kFilterThreads : kScanThreads;
  auto kern = score_scan_kernel<T, D, U, MODE, PAGED, NT, MAXAGG>;
  hipError_t e = hipFuncSetAttribute((const void*)kern, hipFuncAttributeMaxDynamicSharedMemorySize, (int)lds);
  if (e != hipSuccess) return e;
  hipLaunchKernelGGL(kern, grid, dim3(NT), lds, st, a);
  return hipGetLastError();
}

// The filter route is a sum-aggregation path only (its plan is not made for REATTN_AGG_MAX).
template <typename T, int D, int MODE, bool PAGED>
hipError_t launch_hp(const ScanArgs& a, dim3 grid, hipStream_t st) {
  if (MODE != kOutFilter && a.agg_max) return launch_hpa<T, D, MODE == kOutFilter ? kOutScores : MODE, PAGED, true>(a, grid, st);
  return launch_hpa<T, D, MODE, PAGED, false>(a, grid, st);
}

template <typename T, int D>
hipError_t launch_t(const ScanArgs& a, dim3 grid, int mode, hipStream_t st) {
  if (a.pt) return mode == kOutFilter ? launch_hp<T, D, kOutFilter, true>(a, grid, st)
                 : mode == kOutHist   ? launch_hp<T, D, kOutHist, true>(a, grid, st)
                                      : launch_hp<T, D, kOutScores, true>(a, grid, st);
  return mode == kOutFilter ? launch_hp<T, D, kOutFilter, false>(a, grid, st)
       : mode == kOutHist   ? launch_hp<T, D, kOutHist, false>(a, grid, st)
                            : launch_hp<T, D, kOutScores, false>(a, grid, st);
}

}  // namespace

// Rows per workgroup: the whole job is cut into a multiple of the CU count of equal
// slices (each within one KV head) so that every CU streams the same amount and the
// bursts of score writes fall together at the end of each round.
int scan_rows_per_block(int64_t n_mid, int64_t score_rows, int max_rows) {
  int n_cu = 0, dev = 0;                               // of the current device, asked every time: no state is kept
  if (hipGetDevice(&dev) != hipSuccess ||
      hipDeviceGetAttribute(&n_cu, hipDeviceAttributeMultiprocessorCount, dev) != hipSuccess || n_cu <= 0)
    n_cu = 256;
  return scan_rows_per_block_for(n_mid, score_rows, max_rows, n_cu);
}

int scan_rows_per_block_for(int64_t n_mid, int64_t score_rows, int max_rows, int n_cu) {
  if (max_rows <= 0 || max_rows > kScanMaxRows) max_rows = kScanMaxRows;
  const int64_t total = n_mid * score_rows;
  const int64_t r_min = (total + (int64_t)n_cu * max_rows - 1) / ((int64_t)n_cu * max_rows);
  // A row count that does not divide the chip (40 KV heads of a batch of five on 256 CUs) must not spill a few
  // workgroups into a round of their own: every score row gets floor(workgroups / rows) slices, and of the next few
  // round counts the one with the least (rounds x slice length) wins; a workgroup's fixed start (its query rows,
  // its first loads in flight) is priced like kStartRows rows.
  constexpr int64_t kStartRows = 512;
  int64_t best = 0, best_cost = 0;
  for (int64_t rounds = r_min; rounds < r_min + 4; ++rounds) {
    int64_t per_row = rounds * n_cu / score_rows;                      // workgroups per score row
    if (per_row < 1) per_row = 1;
    int64_t rpb = (n_mid + per_row - 1) / per_row;
    rpb = (rpb + 31) / 32 * 32;
    if (rpb > max_rows) rpb = max_rows;
    if (rpb < 32) rpb = 32;
    const int64_t wgs = (n_mid + rpb - 1) / rpb * score_rows;
    const int64_t cost = (wgs + n_cu - 1) / n_cu * (rpb + kStartRows);
    if (best == 0 || cost < best_cost) { best = rpb; best_cost = cost; }
  }
  return (int)best;
}

hipError_t launch_score_scan(const Plan& pl, const void* q, int n_query, const void* k_cache,
                             float* scores, uint32_t* hist, hipStream_t st, const AppendJob* append) {
  if (pl.n_mid <= 0 || n_query <= 0)
    return append ? launch_cache_append(pl, append->first_tok, append->n_tok, append->k_new, append->v_new,
                                        append->k_cache, append->v_cache, st)
                  : hipSuccess;
  ScanArgs a;
  a.ap = append_args(pl, append);
  a.k = k_cache; a.q = q; a.scores = scores; a.hist = hist;
  a.ksh = pl.ksh; a.kst = pl.kst; a.n_mid = pl.n_mid; a.first_tok = pl.s_eff;
  a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.G = pl.G; a.pt = pl.pt; a.page_lg = pl.page_lg;
  a.agg_max = pl.agg == kAggMax ? 1 : 0;
  // max aggregation keeps G * D floats of query rows in LDS behind the parked scores
  a.rows_per_block = scan_rows_per_block(pl.n_mid, (int64_t)pl.Hkv * n_query, a.agg_max ? kScanMaxRows - 4096 : 0);
  dim3 grid((unsigned)((pl.n_mid + a.rows_per_block - 1) / a.rows_per_block),
            (unsigned)(pl.Hkv * n_query));
  a.stream_out = (int64_t)grid.x * grid.y > 320 ? 1 : 0;   // more workgroups than one round over the chip
  a.samp = nullptr; a.samp_stride = 0; a.n_samp = 0; a.rho = 0; a.cand = nullptr; a.segcnt = nullptr;
  const int h = hist != nullptr ? kOutHist : kOutScores;
  if (pl.dtype == kF32) return pl.D == 64 ? launch_t<float, 64>(a, grid, h, st)
                                          : launch_t<float, 128>(a, grid, h, st);
  if (pl.dtype == kF16) return pl.D == 64 ? launch_t<f16bits, 64>(a, grid, h, st)
                                          : launch_t<f16bits, 128>(a, grid, h, st);
  return pl.D == 64 ? launch_t<uint16_t, 64>(a, grid, h, st)
                    : launch_t<uint16_t, 128>(a, grid, h, st);
}

hipError_t launch_score_scan_filter(const Plan& pl, const void* q, const void* k_cache, const float* samp,
                                    uint2* cand, uint32_t* segcnt, hipStream_t st, const AppendJob* append) {
  if (!pl.filter || pl.f_nsamp > (uint32_t)kFilterSampMax || pl.f_rpb > 32 * kFilterThreads) return hipErrorInvalidValue;
  ScanArgs a;
  a.ap = append_args(pl, append);
  a.k = k_cache; a.q = q; a.scores = nullptr; a.hist = nullptr;
  a.ksh = pl.ksh; a.kst = pl.kst; a.n_mid = pl.n_mid; a.first_tok = pl.s_eff;
  a.Hq = pl.Hq; a.Hkv = pl.Hkv; a.G = pl.G; a.pt = pl.pt; a.page_lg = pl.page_lg;
  a.rows_per_block = pl.f_rpb; a.stream_out = 0; a.agg_max = 0;
  a.samp = samp; a.samp_stride = pl.f_samp_stride; a.n_samp = pl.f_nsamp; a.rho = pl.f_rho;
  a.cand = cand; a.segcnt = segcnt;
  const dim3 grid((unsigned)pl.f_nb, (unsigned)pl.Hkv);
  if (pl.dtype == kF32) return pl.D == 64 ? launch_t<float, 64>(a, grid, kOutFilter, st)
                                          : launch_t<float, 128>(a, grid, kOutFilter, st);
  if (pl.dtype == kF16) return pl.D == 64 ? launch_t<f16bits, 64>(a, grid, kOutFilter, st)
                                          : launch_t<f16bits, 128>(a, grid, kOutFilter, st);
  return pl.D == 64 ? launch_t<uint16_t, 64>(a, grid, kOutFilter, st)
                    : launch_t<uint16_t, 128>(a, grid, kOutFilter, st);
}

hipError_t launch_read_probe(const void* buf, size_t bytes, hipStream_t st) {
  const size_t n_vec = bytes / 16;
  if (n_vec == 0) return hipSuccess;
  // up to 8 MiB per workgroup, as in the scan; small buffers are cut finer so that they still fill the chip
  // (a workgroup's waves take 8192 vectors per round)
  size_t vpb = (size_t)kScanMaxRows * 16;
  const size_t even = ((n_vec + 1023) / 1024 + 8191) / 8192 * 8192;
  if (even < vpb) vpb = even;
  hipLaunchKernelGGL(read_probe_kernel, dim3((unsigned)((n_vec + vpb - 1) / vpb)), dim3(kScanThreads),
                     0, st, (const u32x4*)buf, n_vec, vpb, (uint32_t*)nullptr);
  return hipGetLastError();
}

}  // namespace reattn
